"""Pins of the oracle's per-part strategy rule (Sec. 4.2: parts are switched separately; Sec. 4.3: the
smallest inputs want only the MLP intermediate GEMM in INT4, large ones all four parts)."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2301_12017_amd import synth


def _costs(i8, i4, fused):
    return [[a, b] for a, b in zip(i8, i4)], fused


def test_paper_small_input_pattern_gives_q3_only():
    # INT4 pays only for the MLP intermediate GEMM; handing codes over is no cheaper than not
    part, fused = _costs([10, 5, 20, 20], [12, 6, 15, 24], 45)
    assert oracle.pick_strategy(part, fused) == 1 << oracle.PART_FFN1


def test_paper_large_input_pattern_gives_all_parts():
    part, fused = _costs([100, 40, 130, 130], [70, 30, 90, 95], 170)
    assert oracle.pick_strategy(part, fused) == 31          # all four in INT4 and the pair fused
    assert oracle.pick_strategy(part, 190) == 15            # fusing costs more than it saves: not fused


def test_ties_prefer_more_int4_parts_then_the_fused_pair():
    part, fused = _costs([1, 1, 1, 1], [1, 1, 1, 1], 2)
    assert oracle.pick_strategy(part, fused) == 31
    assert oracle.pick_strategy(part, 2.5) == 15


def test_fused_flag_needs_both_ffn_parts():
    for s in range(32):
        both = (s & 12) == 12
        assert oracle.strategy_valid(s) == (not (s & 16) or both)
    with pytest.raises(ValueError):
        oracle.strategy_cost([[1, 1]] * 4, 1, 16 | 4)


def test_pick_equals_the_separable_optimum():
    # QKV and attention output are independent minima; the pair is the least of its five options
    rng = np.random.default_rng(5)
    for _ in range(300):
        part = rng.integers(1, 50, size=(4, 2)).astype(float).tolist()
        fused = float(rng.integers(2, 100))
        s = oracle.pick_strategy(part, fused)
        want = min(part[0]) + min(part[1]) + min(min(a + b for a, b in itertools.product(part[2], part[3])), fused)
        assert oracle.strategy_cost(part, fused, s) == want
        # no other strategy of equal cost has more INT4 parts
        for t in range(32):
            if oracle.strategy_valid(t) and oracle.strategy_cost(part, fused, t) == want:
                assert bin(t & 15).count("1") <= bin(s & 15).count("1")


def test_part_linear_tracks_the_unquantized_layer_better_in_int8():
    # the same part in both precisions against the fp64 product of the fp16 operands: INT8 is the
    # "higher-bit type" of Sec. 4.2, so its error must be the smaller one
    X = synth.activations(24, 128, seed=11)
    W = synth.weights(40, 128, seed=11)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    e4 = np.abs(oracle.part_linear(X, W, True).astype(np.float64) - ref).mean()
    e8 = np.abs(oracle.part_linear(X, W, False).astype(np.float64) - ref).mean()
    assert e8 < e4 / 4 and e4 < 0.5 * np.abs(ref).mean()


def test_ffn_fused_differs_from_unfused_only_by_the_fp16_rounding_of_the_intermediate():
    X = synth.activations(16, 128, seed=12)
    W1, W2 = synth.weights(256, 128, seed=12, tensor_id=1), synth.weights(128, 256, seed=12, tensor_id=3)
    b1, b2 = synth.bias(256, seed=12, tensor_id=2), synth.bias(128, seed=12, tensor_id=4)
    fused = oracle.ffn(X, W1, b1, oracle.ACT_GELU, W2, b2, 31).astype(np.float64)
    plain = oracle.ffn(X, W1, b1, oracle.ACT_GELU, W2, b2, 15).astype(np.float64)
    i8 = oracle.ffn(X, W1, b1, oracle.ACT_GELU, W2, b2, 0).astype(np.float64)
    rms = np.sqrt((i8 ** 2).mean())
    assert np.abs(fused - plain).max() < 0.25 * rms          # a few codes of the intermediate flip, no more
    assert np.sqrt(((plain - i8) ** 2).mean()) < 0.5 * rms   # both precisions compute the same layer
