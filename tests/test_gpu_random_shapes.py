"""Seeded random shapes through the one-launch small-token path, the INT8 sibling and the LayerNorm
kernel: ragged M, N, K inside each entry point's contract, all in one process."""
import numpy as np
import pytest

from tests.gpu_util import GELU_SAME, OLAY_SAME, assert_f16, dev, f16_close, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


def test_small_token_path_random_shapes(B, orc):
    rng = np.random.default_rng(2024)
    for _ in range(24):
        M = int(rng.integers(1, 200))
        N = 8 * int(rng.integers(1, 80))
        K = 64 * int(rng.integers(1, 65))
        act = int(rng.integers(0, 2))
        X = rng.standard_normal((M, K)).astype(np.float32).astype(np.float16)
        W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
        b = (rng.standard_normal(N) * 0.01).astype(np.float16) if rng.integers(0, 2) else None
        Q = B.quantize_weight(dev(W), 0)
        got = host(B.linear_f16act(dev(X), Q, None if b is None else dev(b), act))
        want = orc.linear(orc.quantize_act(X, 0), orc.quantize_weight(W, 0), 0, 0, b, act)["out"]
        ok, ratio = f16_close(got, want)
        assert ok, (M, N, K, act, ratio)
        if act == 0:
            assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), (M, N, K)


def test_int8_sibling_random_shapes(B, orc):
    rng = np.random.default_rng(2025)
    for _ in range(16):
        M = int(rng.integers(1, 700))
        N = 8 * int(rng.integers(1, 90))
        K = 64 * int(rng.integers(2, 40))
        X = rng.standard_normal((M, K)).astype(np.float32).astype(np.float16)
        W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
        b = (rng.standard_normal(N) * 0.01).astype(np.float16)
        Aq, sa = B.quantize_rows8(dev(X))
        Wq, sw = B.quantize_rows8(dev(W))
        rows = np.sort(rng.choice(M, min(M, 48), replace=False))
        a, w = orc.quantize_rows8(X[rows]), orc.quantize_rows8(W)
        assert np.array_equal(host(Aq)[rows], a["q"]) and np.array_equal(host(Wq), w["q"])
        assert np.array_equal(host(B.gemm8_i32(Aq, sa, Wq, sw))[rows], orc.gemm8_i32(a["q"], w["q"])), (M, N, K)
        got = host(B.linear8(Aq, sa, Wq, sw, dev(b), 0))[rows]
        assert np.array_equal(got.view(np.uint16), orc.linear8(a, w, b, 0)["out"].view(np.uint16)), (M, N, K)


def test_layernorm_random_shapes(B, orc):
    rng = np.random.default_rng(2026)
    for _ in range(16):
        M = int(rng.integers(1, 300))
        K = 32 * int(rng.integers(1, 129))
        mode = int(rng.integers(0, 2))
        x = (rng.standard_normal((M, K)) * rng.uniform(0.1, 5)).astype(np.float32).astype(np.float16)
        r = rng.standard_normal((M, K)).astype(np.float16) if rng.integers(0, 2) else None
        g = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
        b = (0.1 * rng.standard_normal(K)).astype(np.float16)
        want = orc.layernorm_quantize(x, r, g, b, 1e-5, mode)
        A, y = B.layernorm_quantize(dev(x), None if r is None else dev(r), dev(g), dev(b), 1e-5, mode)
        np.testing.assert_allclose(host(A.scale), want["s"], rtol=1e-5)
        gc = orc.unpack(host(A.q), mode).astype(np.int32)
        wc = orc.unpack(want["q"], mode).astype(np.int32)
        assert np.max(np.abs(gc - wc)) <= 1 and np.mean(gc != wc) <= 2e-3, (M, K, mode)
        yy, wy = host(y).astype(np.float64), want["y16"].astype(np.float64)
        assert np.all(np.abs(yy - wy) <= np.maximum(np.abs(wy) * 2.0 ** -10, 2.0 ** -24)), (M, K, mode)


def test_operand_layout_gemm_random_shapes(B, orc):
    """The persistent kernel (both tiles) on ragged M and N: int32 sums and fp16 outputs of sampled rows."""
    from tests.gpu_util import act_to_canonical, olay_schedules, wgt_to_canonical
    rng = np.random.default_rng(2027)
    for _ in range(10):
        M = int(rng.integers(1, 2500))
        N = 8 * int(rng.integers(1, 160))
        K = 128 * int(rng.integers(2, 17))
        X = rng.standard_normal((M, K)).astype(np.float32).astype(np.float16)
        W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
        b = (rng.standard_normal(N) * 0.01).astype(np.float16)
        A = B.quantize_act(dev(X), 0, layout=1)
        Q = B.quantize_weight(dev(W), 0, layout=1)
        rows = np.sort(rng.choice(M, min(M, 40), replace=False))
        oa, ow = orc.quantize_act(X[rows], 0), orc.quantize_weight(W, 0)
        assert np.array_equal(act_to_canonical(host(A.q))[rows], oa["q"]) and np.array_equal(wgt_to_canonical(host(Q.q)), ow["q"])
        wantP = orc.gemm_i32(oa["q"], ow["q"], 0, 0)
        want = orc.linear(oa, ow, 0, 0, b, 0)["out"]
        for sch in olay_schedules(B, K):
            assert np.array_equal(host(B.gemm_i32(A, Q, schedule=sch))[:, rows], wantP), (M, N, K, sch)
            got = host(B.linear(A, Q, dev(b), 0, schedule=sch))[rows]
            assert_f16(got, want, OLAY_SAME if got.size > 4000 else 0.98, str((M, N, K, sch)))


def test_fp6_path_random_shapes(B, orc):
    """The FP6 path on ragged M and N and every K the layout is offered for up to 4096: int32 sums of sampled rows on
    every tile, fp16 outputs bit for bit, and - where N is a multiple of 256 - the fused requantize into the FP6 layout
    (codes and scales bit for bit)."""
    from tests.gpu_util import fp6_plan, fp6_schedules, fp6_to_codes
    rng = np.random.default_rng(2028)
    done = 0
    while done < 10:
        M = int(rng.integers(1, 1500))
        K = 256 * int(rng.integers(2, 17))
        if fp6_plan(K) is None:
            continue
        requant = bool(rng.integers(0, 2))
        N = 256 * int(rng.integers(1, 7)) if requant else 8 * int(rng.integers(1, 130))
        done += 1
        X = (rng.standard_normal((M, K)) * rng.uniform(0.2, 3.0, size=(M, 1))).astype(np.float32).astype(np.float16)
        W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
        b = (rng.standard_normal(N) * 0.01).astype(np.float16)
        A, Q = B.quantize_act(dev(X), 0, layout=2), B.quantize_weight(dev(W), 0, 0, layout=2)
        rows = np.sort(rng.choice(M, min(M, 40), replace=False))
        a, w = orc.quantize_act(np.ascontiguousarray(X[rows]), 0), orc.quantize_weight(W, 0, 0)
        want = orc.gemm_i32(a["q"], w["q"], 0, 0)
        for sch in fp6_schedules(B, K):
            got = host(B.gemm_i32(A, Q, schedule=sch)).reshape(M, N)[rows]
            assert np.array_equal(got, want.reshape(len(rows), N)), (M, N, K, B.schedule_names()[sch - 1])
        y = host(B.linear(A, Q, dev(b), 0))[rows]
        assert np.array_equal(y.view(np.uint16), orc.linear(a, w, 0, 0, b, 0)["out"].view(np.uint16)), (M, N, K)
        if requant:
            out = B.linear(A, Q, dev(b), 0, requant=True, requant_layout=2)
            ref = orc.linear(a, w, 0, 0, b, 0, requant=True, requant_mode=0, requant_group=0)
            assert np.array_equal(host(out.scale)[rows].view(np.uint32), ref["s"].view(np.uint32)), (M, N, K)
            codes = fp6_to_codes(host(out.q), N, M)[rows]
            assert np.array_equal(codes, orc.unpack(ref["q"], 0)), (M, N, K)
    assert B.fused_fault_check() is False
