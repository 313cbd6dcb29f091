"""Pins for the oracle's quantizers (Sec. 3.1 symmetric / asymmetric mapping,
App. A token-wise activations and group-wise weights).

None of these re-type the oracle's formula: they check closed forms, the
half-step error bound, exact rational arithmetic, invariants and the tie rule.
"""
import numpy as np
import pytest


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("e", [-20, -3, 0, 5])
def test_sym_closed_form_power_of_two_grid(orc, e):
    c = np.float32(2.0 ** e)
    v = (np.arange(-7, 8, dtype=np.float32) * c)
    q, S = orc.quant_sym(v)
    assert S == c
    assert list(q) == list(range(-7, 8))


def test_sym_absmax_maps_to_plus_minus_seven(orc):
    rng = np.random.default_rng(3)
    for _ in range(200):
        v = rng.standard_normal(96).astype(np.float32) * np.float32(rng.uniform(1e-3, 50))
        q, S = orc.quant_sym(v)
        i = int(np.argmax(np.abs(v)))
        assert abs(int(q[i])) == 7 and np.sign(q[i]) == np.sign(v[i])
        assert q.min() >= -7 and q.max() <= 7          # -8 never produced with S = absmax/7
        assert S == np.float32(np.abs(v).max()) / np.float32(7.0)


@pytest.mark.parametrize("lo,step", [(-3.0, 0.25), (0.5, 2.0 ** -6), (-1024.0, 64.0)])
def test_asym_closed_form_grid(orc, lo, step):
    v = (np.float32(lo) + np.float32(step) * np.arange(16, dtype=np.float32))
    v = v[np.random.default_rng(0).permutation(16)]
    q, S, Z = orc.quant_asym(v)
    assert Z == np.float32(lo)
    assert S == np.float32(step)
    assert np.array_equal(q.astype(np.float32), (v - np.float32(lo)) / np.float32(step))


def test_asym_min_is_zero_max_is_fifteen(orc):
    rng = np.random.default_rng(4)
    for _ in range(200):
        v = (rng.standard_normal(128) * rng.uniform(0.01, 30) + rng.uniform(-5, 5)).astype(np.float32)
        q, S, Z = orc.quant_asym(v)
        assert Z == v.min()
        assert q[np.argmin(v)] == 0 and q[np.argmax(v)] == 15
        assert q.min() >= 0 and q.max() <= 15


def test_degenerate_vectors(orc):
    q, S = orc.quant_sym(np.zeros(32, np.float32))
    assert S == 1.0 and not q.any()
    q, S, Z = orc.quant_asym(np.full(32, 2.5, np.float32))
    assert S == 1.0 and Z == 2.5 and not q.any()


# ---------------------------------------------------------------- error bound
def _heavy(rng, n):
    v = rng.standard_normal(n).astype(np.float32)
    v[rng.choice(n, 4, replace=False)] *= 20
    return v


def test_error_at_most_half_a_step(orc):
    rng = np.random.default_rng(5)
    slack = 1 + 2.0 ** -20
    for trial in range(300):
        v = _heavy(rng, 256) if trial % 2 else rng.standard_normal(256).astype(np.float32)
        q, S = orc.quant_sym(v)
        err = np.abs(v.astype(np.float64) - np.float64(S) * q)
        assert err.max() <= 0.5 * float(S) * slack
        q, S, Z = orc.quant_asym(v)
        err = np.abs(v.astype(np.float64) - (np.float64(S) * q + np.float64(Z)))
        assert err.max() <= 0.5 * float(S) * slack


# ---------------------------------------------------------------- exact arithmetic
def _exact_rne_ratio(num, den):
    """round-half-even of num/den for positive python/numpy integers; also flags ties."""
    fl = num // den
    rem2 = 2 * (num - fl * den)
    up = (rem2 > den) | ((rem2 == den) & (fl % 2 == 1))
    return fl + up, rem2 == den


def test_sym_codes_equal_exact_rational_rounding_off_ties(orc):
    """For fp16 inputs, rne(x * (7/amax)) in fp32 equals exact round-half-even of
    7x/amax whenever 7x/amax is not exactly a half-integer (checked with integers)."""
    rng = np.random.default_rng(6)
    allpos = np.arange(1, 0x7C00, dtype=np.uint16)                  # all positive finite fp16
    scale = 2 ** 24                                                 # fp16 values are integers / 2^24
    ints = (allpos.view(np.float16).astype(np.float64) * scale).astype(np.int64)
    for amax_bits in rng.choice(allpos[allpos > 0x0400], 60, replace=False):
        amax_i = int(np.float64(np.uint16(amax_bits).view(np.float16)) * scale)
        sel = ints <= amax_i
        xs = allpos[sel].view(np.float16).astype(np.float32)
        v = np.concatenate([xs, [np.float32(np.uint16(amax_bits).view(np.float16))]]).astype(np.float32)
        q, _ = orc.quant_sym(v)
        want, tie = _exact_rne_ratio(7 * ints[sel].astype(object), amax_i)
        want = np.array(want, dtype=np.int64)
        tie = np.array(tie, dtype=bool)
        got = q[:-1].astype(np.int64)
        assert np.array_equal(got[~tie], want[~tie])
        assert np.all(np.abs(got[tie] - want[tie]) <= 1)


def test_ties_round_to_even(orc):
    # amax = 7 -> inv = 1 exactly, so the codes are rne of the inputs themselves.
    v = np.array([7, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 6.5, -6.5, 0.49, 0.51], np.float32)
    q, S = orc.quant_sym(v)
    assert S == 1.0
    assert list(q) == [7, 0, 2, 2, 4, 0, -2, -2, 6, -6, 0, 1]
    v = np.array([0, 15, 0.5, 1.5, 2.5, 13.5, 14.5], np.float32)
    q, S, Z = orc.quant_asym(v)
    assert S == 1.0 and Z == 0.0
    assert list(q) == [0, 15, 0, 2, 2, 14, 14]


def test_clamp_guards_range(orc):
    # The clamp is only a guard under S = absmax/7; feed the internal range directly:
    # a vector whose scaled values would exceed the code range cannot be built through
    # quant_sym (absmax defines the range), so check the unsigned upper edge instead.
    v = np.array([0.0, 1.0, np.nextafter(np.float32(1.0), np.float32(2.0))], np.float32)
    q, S, Z = orc.quant_asym(v)
    assert q.max() == 15 and q.min() == 0


# ---------------------------------------------------------------- invariants
def test_power_of_two_scaling_invariance(orc):
    rng = np.random.default_rng(7)
    v = rng.standard_normal(200).astype(np.float32)
    q0, S0 = orc.quant_sym(v)
    a0, T0, Z0 = orc.quant_asym(v)
    for e in (-10, -1, 3, 12):
        f = np.float32(2.0 ** e)
        q, S = orc.quant_sym(v * f)
        assert np.array_equal(q, q0) and S == S0 * f
        a, T, Z = orc.quant_asym(v * f)
        assert np.array_equal(a, a0) and T == T0 * f and Z == Z0 * f


def test_negation_symmetry_off_ties(orc):
    v = np.random.default_rng(8).standard_normal(500).astype(np.float32)
    q, S = orc.quant_sym(v)
    qn, Sn = orc.quant_sym(-v)
    assert S == Sn and np.array_equal(qn, -q)


def test_idempotence_on_dequantized_values(orc):
    rng = np.random.default_rng(9)
    for _ in range(50):
        q = rng.integers(-7, 8, 64).astype(np.int8)
        q[0] = 7
        S = np.float32(2.0 ** rng.integers(-8, 8))          # exact products
        q2, S2 = orc.quant_sym(q.astype(np.float32) * S)
        assert S2 == S and np.array_equal(q2, q)
        u = rng.integers(0, 16, 64).astype(np.uint8)
        u[0], u[1] = 0, 15
        zero = np.float32(rng.integers(-64, 64)) * S
        u2, S3, Z3 = orc.quant_asym(u.astype(np.float32) * S + zero)
        assert S3 == S and Z3 == zero and np.array_equal(u2, u)


# ---------------------------------------------------------------- row / group drivers
def test_quantize_act_is_rowwise_and_packs(orc):
    rng = np.random.default_rng(10)
    X = rng.standard_normal((9, 256)).astype(np.float16)
    for mode in (orc.SYM, orc.ASYM):
        A = orc.quantize_act(X, mode, group=128)
        codes = orc.unpack(A["q"], mode)
        for m in range(9):
            row = X[m].astype(np.float32)
            if mode == orc.SYM:
                q, S = orc.quant_sym(row)
                assert A["z"][m] == 0
            else:
                q, S, Z = orc.quant_asym(row)
                assert A["z"][m] == Z
            assert A["s"][m] == S
            assert np.array_equal(codes[m].astype(np.int16), q.astype(np.int16))
        want = codes.astype(np.int32).reshape(9, 2, 128).sum(-1)
        assert np.array_equal(A["gsum"], want)


def test_quantize_weight_groups_are_independent_vectors(orc):
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((6, 384)) * 0.02).astype(np.float16)
    for mode in (orc.SYM, orc.ASYM):
        for group in (0, 128):
            Q = orc.quantize_weight(W, mode, group)
            G = 384 if group == 0 else group
            ng = 384 // G
            codes = orc.unpack(Q["q"], mode)
            for n in range(6):
                for g in range(ng):
                    seg = W[n, g * G:(g + 1) * G].astype(np.float32)
                    if mode == orc.SYM:
                        q, S = orc.quant_sym(seg)
                        Z = np.float32(0)
                    else:
                        q, S, Z = orc.quant_asym(seg)
                    assert Q["s"][n, g] == S and Q["z"][n, g] == Z
                    assert np.array_equal(codes[n, g * G:(g + 1) * G].astype(np.int16), q.astype(np.int16))
                    assert Q["gsum"][n, g] == int(q.astype(np.int64).sum())
            # c[n] is the sum over k of the dequantized weight
            wh = orc.dequantize_operand(Q["q"], mode, Q["s"], Q["z"])
            # (fp32 sums of terms of size K*|zero| ~ 25 cancel: absolute floor ~ 25 * 2^-23)
            np.testing.assert_allclose(Q["c"], wh.sum(1), rtol=2e-6, atol=5e-6)


def test_quantization_noise_level_gaussian(orc):
    """Statistical sanity, not parity: a uniform 4-bit grid over +-absmax of a Gaussian
    row has step ~ 2*absmax/14 and noise step/sqrt(12): about 10-17 % of sigma at K=768."""
    X = np.random.default_rng(12).standard_normal((64, 768)).astype(np.float16)
    A = orc.quantize_act(X, orc.SYM)
    xh = orc.dequantize_operand(A["q"], orc.SYM, A["s"])
    rel = np.linalg.norm(xh - X.astype(np.float64)) / np.linalg.norm(X.astype(np.float64))
    assert 0.08 < rel < 0.2
