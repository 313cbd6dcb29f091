"""Pins for the oracle's fp16 conversions and nibble packing.

fp16: checked against numpy's IEEE binary16 (an implementation the oracle does
not use).  Packing (Sec. 4.2: INT4 data carried inside INT8 tensors): checked
against the byte examples stored in tests/golden/pack_examples.txt, against an
independent bit-twiddling unpack written here, and by round trip.
"""
import os

import numpy as np

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_h2f_all_bit_patterns(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([orc.h2f(int(b)) for b in bits], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f2h_matches_ieee_rounding(orc):
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0),
        (rng.standard_normal(5000) * 1e-6).astype(np.float32),          # fp16 subnormal range
        (rng.standard_normal(5000) * 3e4).astype(np.float32),           # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0**-24, 2.0**-25,
                  1.5 * 2.0**-24, 2.5 * 2.0**-24, 2.0**-14, 1.0 + 2.0**-11, 1.0 + 3 * 2.0**-11,
                  2047.5 * 2.0**-10 * 2.0], np.float32),
    ])
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([orc.f2h(float(v)) for v in vals], np.uint16)
    assert np.array_equal(got, want)


def test_store_f16_vector(orc):
    y = np.random.default_rng(2).standard_normal((7, 33)).astype(np.float32)
    assert np.array_equal(orc.store_f16(y).view(np.uint16), y.astype(np.float16).view(np.uint16))


def _golden_pack_examples():
    rows = []
    with open(os.path.join(GOLD, "pack_examples.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                mode, lo, hi, byte = line.split()
                rows.append((mode, int(lo), int(hi), int(byte, 16)))
    return rows


def test_pack_golden_bytes(orc):
    rows = _golden_pack_examples()
    assert len(rows) >= 3
    for mode, lo, hi, byte in rows:
        got = orc.pack(np.array([lo, hi], np.int8))
        assert got[0] == byte, (mode, lo, hi, hex(got[0]))


def _unpack_independent(packed, signed):
    lo = (packed & 0xF).astype(np.int16)
    hi = (packed >> 4).astype(np.int16)
    if signed:
        lo = np.where(lo > 7, lo - 16, lo)
        hi = np.where(hi > 7, hi - 16, hi)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), np.int16)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


def test_unpack_all_bytes_and_round_trip(orc):
    allb = np.arange(256, dtype=np.uint8)[None, :]
    for mode, signed in ((orc.SYM, True), (orc.ASYM, False)):
        codes = orc.unpack(allb, mode)
        assert np.array_equal(codes.astype(np.int16), _unpack_independent(allb, signed))
        assert np.array_equal(orc.pack(codes.reshape(-1)), allb.reshape(-1))
        lo_rng = (-8, 8) if signed else (0, 16)
        for a in range(*lo_rng):
            for b in range(*lo_rng):
                by = orc.pack(np.array([a, b], np.int8))
                back = orc.unpack(by[None, :], mode)[0]
                assert (int(back[0]), int(back[1])) == (a, b)


def test_pack_order_is_low_nibble_first(orc):
    codes = np.array([1, 2, 3, 4, -1, -2, 7, -8], np.int8)
    assert list(orc.pack(codes)) == [0x21, 0x43, 0xEF, 0x87]
