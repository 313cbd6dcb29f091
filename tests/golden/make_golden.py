"""Writes tests/golden/config1_oracle_digest.json: SHA-256 digests of what the CPU
oracle computes for workload 1 (one 128 x 768 x 768 symmetric W4A4 linear, seed 0).

The paper prints no worked numeric example for the quantizer or the GEMM, so this
file is a regression guard for the oracle, not an external pin: it records the
oracle's own results (the external pins are the closed-form / brute-force /
float64 tests).  It calls only oracle/ and the seeded input generator.

Run from the repository root:  python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import oracle  # noqa: E402
from paper_2301_12017_amd import synth  # noqa: E402


def digests():
    spec = synth.config_linears(1)[0]
    X, W, b = synth.linear_inputs(spec, 1, 0)
    A = oracle.quantize_act(X, oracle.SYM)
    Q = oracle.quantize_weight(W, oracle.SYM)
    P = oracle.gemm_i32(A["q"], Q["q"], oracle.SYM)
    res = oracle.linear(A, Q, oracle.SYM, 0, b, oracle.ACT_NONE)

    def h(a):
        return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()

    return {
        "workload": "config 1: M=128 K=768 N=768, symmetric, per-channel, bias, seed 0",
        "X_f16": h(X), "W_f16": h(W), "bias_f16": h(b),
        "Aq": h(A["q"]), "sa": h(A["s"]), "Wq": h(Q["q"]), "sw": h(Q["s"]),
        "P_i32": h(P), "Y_f16": h(res["out"]),
        "P_sum": int(P.astype(np.int64).sum()), "P_absmax": int(np.abs(P).max()),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config1_oracle_digest.json")
    with open(out, "w") as f:
        json.dump(digests(), f, indent=1)
        f.write("\n")
    print("wrote", out)
