"""Every fp16 (absmax, x) pair of the symmetric mapping (Sec. 3.1, b = 4), enumerated on the CPU.

The definition is code = rne(clamp(x * (7 / absmax), -8, 7)) in fp32.  The kernels take the same product and
round it by adding 1.5 * 2^23 + 8 (the fp32 add rounds to nearest even) and reading the low four bits of the sum
(offset binary, code + 8), without the clamp.  Two things make that the same decision for every input an fp16
activation tensor can hold, and both are checked here over ALL finite positive fp16 absmax values and ALL fp16
x with |x| <= absmax, both signs (5.0e8 pairs):
  * the clamp cannot bind: |x * inv| <= 7 * (1 + 2^-23) < 7.5, so the rounded code stays inside [-7, 7];
  * the magic-number rounding equals rne of the product, also on exact ties (k + 0.5), which occur: they are
    counted, and there must be some for the test to mean anything.
The oracle's own routine is cross-checked against the same enumeration on a sample of absmax values.
"""
import numpy as np


def _all_positive_fp16():
    bits = np.arange(1, 0x7C00, dtype=np.uint16)               # every positive finite fp16, subnormals included
    return bits.view(np.float16).astype(np.float32)


def test_symmetric_codes_every_fp16_pair():
    vals = _all_positive_fp16()                                 # ascending
    seven = np.float32(7.0)
    magic = np.float32(12582920.0)                              # 1.5 * 2^23 + 8
    ties = pairs = 0
    worst = 0.0
    block = 64
    for b0 in range(0, len(vals), block):
        amax = vals[b0:b0 + block][:, None]                     # [B, 1]
        x = vals[None, :b0 + block]                             # candidates; masked to x <= amax below
        inv = (seven / amax).astype(np.float32)
        t = (x * inv).astype(np.float32)                        # one fp32 multiply, as both sides do
        valid = x <= amax
        # definition (positive and negative x: t and -t)
        for sign in (1.0, -1.0):
            ts = (t * np.float32(sign)).astype(np.float32)
            want = np.rint(np.clip(ts, np.float32(-8.0), np.float32(7.0))).astype(np.int32)
            u = (ts + magic).astype(np.float32)
            got = (u.view(np.uint32) & 0xF).astype(np.int32) - 8
            bad = valid & (got != want)
            assert not bad.any(), (float(amax[np.argwhere(bad)[0][0], 0]), float(x[0, np.argwhere(bad)[0][1]]))
        frac = t - np.floor(t)
        ties += int((valid & (frac == np.float32(0.5))).sum())
        pairs += int(valid.sum())
        worst = max(worst, float(t[valid].max()))
    assert pairs > 4.9e8
    assert worst <= 7.0 * (1 + 2.0 ** -23)                      # the clamp never binds
    assert ties > 1000                                          # exact ties exist and were all decided alike
    print(f"pairs {2 * pairs}, exact ties {2 * ties}, largest |x*inv| = 7*(1+{worst / 7.0 - 1:.3e})")


def test_oracle_routine_agrees_on_sampled_absmax(orc):
    """The oracle's quantize_act on rows that hold one absmax and a sweep of all smaller fp16 values."""
    vals = _all_positive_fp16()
    rng = np.random.default_rng(7)
    picks = np.concatenate([[len(vals) - 1, 1023, 1024, 15360], rng.choice(len(vals), 60, replace=False)])
    seven = np.float32(7.0)
    for idx in picks:
        amax = vals[idx]
        xs = vals[:idx + 1]
        row = np.concatenate([xs, -xs]).astype(np.float16)
        if len(row) % 2:
            row = np.concatenate([row, row[:1]])
        out = orc.quantize_act(row[None, :], 0, 0)
        codes = orc.unpack(out["q"], 0)[0].astype(np.int32)
        inv = seven / amax
        t = (row.astype(np.float32) * inv).astype(np.float32)
        want = np.rint(np.clip(t, -8.0, 7.0)).astype(np.int32)
        assert np.array_equal(codes, want), float(amax)
        assert out["s"][0] == np.float32(amax) / seven
