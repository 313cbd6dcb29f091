"""Host logic of the per-part strategy (Sec. 4.2: parts switched separately; Sec. 4.3: which parts
pay depends on the input size): the library's pick against the oracle's brute force, the built-in
table, and argument errors.  No GPU is touched."""
import ctypes
import os

import numpy as np
import pytest

import oracle


@pytest.fixture(scope="module")
def b():
    from paper_2301_12017_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2301_12017_amd import build
        build.build(verbose=False)
    return binding


def test_pick_matches_the_oracle_on_random_cost_tables(b):
    rng = np.random.default_rng(2)
    for _ in range(2000):
        # small integers: plenty of exact ties, so the tie rules are exercised too
        part = rng.integers(1, 12, size=(4, 2)).astype(float).tolist()
        fused = float(rng.integers(2, 24))
        assert b.strategy_pick(part, fused) == oracle.pick_strategy(part, fused), (part, fused)


def test_pick_matches_the_oracle_on_measured_looking_tables(b):
    rng = np.random.default_rng(3)
    for _ in range(500):
        part = (rng.random((4, 2)) * 200 + 3).astype(np.float32).astype(float).tolist()
        fused = float(np.float32(rng.random() * 400 + 6))
        assert b.strategy_pick(part, fused) == oracle.pick_strategy(part, fused)


def test_pick_reproduces_both_regimes_of_the_paper(b):
    assert b.strategy_pick([[10, 12], [5, 6], [20, 15], [20, 24]], 45) == 1 << b.PART_FFN1
    assert b.strategy_pick([[100, 70], [40, 30], [130, 90], [130, 95]], 170) == b.STRATEGY_ALL_INT4


def test_pick_rejects_bad_costs(b):
    L = b.lib()
    assert L.w4a4_strategy_pick(None) == -1
    for bad in (-1.0, float("nan"), float("inf")):
        c = b._costs_struct([[1, 1]] * 4, 1)
        c.part_us[2][1] = bad
        assert L.w4a4_strategy_pick(ctypes.byref(c)) == -1
        c = b._costs_struct([[1, 1]] * 4, bad)
        assert L.w4a4_strategy_pick(ctypes.byref(c)) == -1


def test_lookup_table_and_shape_errors(b):
    L = b.lib()
    assert b.strategy_lookup(128, 768, 3072) == 15                       # one-kernel parts, not fused
    assert b.strategy_lookup(16384, 768, 3072) == b.STRATEGY_ALL_INT4
    assert b.strategy_lookup(12288, 1024, 4096) == b.STRATEGY_ALL_INT4
    for M, h, f in [(0, 768, 3072), (128, 100, 3072), (128, 768, 3000), (128, 8192, 3072), (128, 768, 32768), (128, 64, 256)]:
        assert L.w4a4_strategy_lookup(M, h, f) == -1
        assert L.w4a4_strategy_tune(M, h, f, 5, None, None) == -1
    assert L.w4a4_strategy_tune(128, 768, 3072, 0, None, None) == -1      # iters


def _part(b, N=64, K=128, act=0, mode=0, w8=0x2000):
    w = b._Weight(0x1000, 0x1000, 0x1000 if mode else None, 0x1000 if mode else None, N, K, 0, mode, 0, None)
    return b._Part(w, w8, w8, None, act)


def test_part_and_ffn_argument_errors(b):
    L = b.lib()
    p = ctypes.c_void_p(0x4000)
    P = _part(b)
    need = L.w4a4_part_workspace_bytes(8, ctypes.byref(P))
    assert need >= 8 * 128 + 8 * 4 and need % 256 == 0
    assert L.w4a4_part_workspace_bytes(0, ctypes.byref(P)) == 0 and L.w4a4_part_workspace_bytes(8, None) == 0

    def run(M=8, ldx=128, part=P, x=p, o=p, ws=p, nbytes=1 << 20, int4=1):
        return L.w4a4_part_linear(x, M, ldx, ctypes.byref(part) if part is not None else None, int4, o, ws, nbytes, None)

    assert run(part=None) == -1 and run(M=-1) == -1 and run(ldx=64) == -1
    assert run(x=None) == -1 and run(o=None) == -1
    assert run(part=_part(b, act=9)) == -1
    assert run(part=_part(b, K=48)) == -1                                  # K % 32
    assert run(ws=None) == -3 and run(nbytes=16) == -3
    assert run(ws=ctypes.c_void_p(0x4010)) == -3                           # workspace not 256-byte aligned
    assert run(part=_part(b, w8=None), int4=0) == -1                       # INT8 form missing
    assert run(M=0) == 0

    F1, F2 = _part(b, N=256, K=128, act=1), _part(b, N=128, K=256)
    wsb = L.w4a4_ffn_workspace_bytes(8, ctypes.byref(F1), ctypes.byref(F2))
    assert wsb >= 8 * 256 * 2
    assert L.w4a4_ffn_workspace_bytes(8, ctypes.byref(F1), ctypes.byref(F1)) == 0      # N1 != K2

    def ffn(strategy, f1=F1, f2=F2, M=8, ws=p, nbytes=1 << 20, x=p, o=p):
        return L.w4a4_ffn(x, M, 128, ctypes.byref(f1), ctypes.byref(f2), strategy, o, ws, nbytes, None)

    assert ffn(16) == -1 and ffn(16 | 4) == -1 and ffn(16 | 8) == -1       # the fused pair needs both parts in INT4
    assert ffn(32) == -1 and ffn(-1) == -1
    assert ffn(12, f2=F1) == -1                                            # shapes do not chain
    assert ffn(28, f2=_part(b, N=128, K=256, mode=1)) == -2                # fused needs symmetric FFN2 weights
    assert ffn(12, ws=None) == -3 and ffn(12, nbytes=64) == -3
    assert ffn(12, x=None) == -1 and ffn(12, o=None) == -1
    assert ffn(12, M=0) == 0


def test_attention_argument_errors(b):
    L = b.lib()
    p = ctypes.c_void_p(0x4000)
    assert L.w4a4_attention_f16(p, -1, 8, 2, p, None) == -1 and L.w4a4_attention_f16(p, 1, 8, 0, p, None) == -1
    assert L.w4a4_attention_f16(None, 1, 8, 2, p, None) == -1 and L.w4a4_attention_f16(p, 1, 8, 2, None, None) == -1
    assert L.w4a4_attention_f16(p, 1, 513, 2, p, None) == -2                # keys and values must fit the LDS
    assert L.w4a4_attention_f16(ctypes.c_void_p(0x4008), 1, 8, 2, p, None) == -2
    assert L.w4a4_attention_f16(p, 0, 8, 2, p, None) == 0 and L.w4a4_attention_f16(p, 3, 0, 2, p, None) == 0


def test_encoder_layer_argument_errors(b):
    L = b.lib()
    p = ctypes.c_void_p(0x4000)
    h, heads, f = 128, 2, 256

    def weights(**kw):
        parts = dict(qkv=_part(b, 3 * h, h), attn_out=_part(b, h, h), ffn1=_part(b, f, h, act=1), ffn2=_part(b, h, f))
        parts.update({k: v for k, v in kw.items() if k in parts})
        return b._LayerWeights(kw.get("hidden", h), kw.get("heads", heads), kw.get("ffn", f), parts["qkv"], parts["attn_out"],
                               parts["ffn1"], parts["ffn2"], kw.get("g1", 0x5000), 0x5000, 0x5000, 0x5000, kw.get("eps", 1e-12))

    W = weights()
    need = L.w4a4_encoder_layer_workspace_bytes(2, 8, ctypes.byref(W))
    assert need >= 16 * (3 * h + 4 * h) * 2 and need % 256 == 0
    assert L.w4a4_encoder_layer_workspace_bytes(0, 8, ctypes.byref(W)) == 0
    assert L.w4a4_encoder_layer_workspace_bytes(2, 8, None) == 0

    def run(strategy=15, w=W, batch=2, seq=8, x=p, o=p, ws=p, nbytes=1 << 24):
        return L.w4a4_encoder_layer(x, batch, seq, ctypes.byref(w), strategy, o, ws, nbytes, None)

    assert run(w=weights(heads=3)) == -1                                     # hidden != heads * 64
    assert run(w=weights(qkv=_part(b, 2 * h, h))) == -1                      # part shapes must chain
    assert run(w=weights(ffn2=_part(b, h, f, mode=1))) == -1                 # symmetric FFN weights
    assert run(w=weights(g1=None)) == -1 and run(w=weights(eps=-1.0)) == -1
    assert L.w4a4_encoder_layer_workspace_bytes(2, 8, ctypes.byref(weights(heads=3))) == 0
    assert run(strategy=64) == -1 and run(strategy=-1) == -1
    assert run(strategy=16 | 4) == -1 and run(strategy=32 | 3) == -1         # flags without their parts
    assert run(x=None) == -1 and run(o=None) == -1
    assert run(seq=600) == -2
    assert run(ws=None) == -3 and run(nbytes=1024) == -3 and run(ws=ctypes.c_void_p(0x4040)) == -3
    assert run(batch=0) == 0
