"""The MFMA operand layout of UNSIGNED codes (asymmetric mapping, weight K-groups) and the group kernel that reads it.

Codes, scales, zero points and code sums must equal the oracle's bit for bit (the layout is a byte-wise bijection of
the canonical bytes, mapped back here with bit operations); the layout-private sums must describe those codes; the
int32 planes must be exact.  fp16 outputs: this kernel evaluates the definition's real number with fused multiply-adds
and in another order, and the unsigned mapping's terms cancel heavily (|sa*t1| is hundreds of times |y| with outlier
channels), so the comparison is the 1e-2 tolerance plus an error budget against the float64 evaluation of the
dequantized operands: the kernel may be no further from it than the oracle's own fp32 evaluation is, up to a factor.
"""
import numpy as np
import pytest
import torch

from tests.gpu_util import (act_to_canonical, asym_budget, dev, f16_close_budget, f16_steps, has_gpu, host, qact_host,
                            qweight_host, wgt_to_canonical)

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]

ASYM, MFMA = 1, 1


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


def _x(rng, M, K, outliers=4):
    x = rng.standard_normal((M, K)).astype(np.float32)
    if outliers:
        x[:, rng.choice(K, outliers, replace=False)] *= 20.0
    return x.astype(np.float16)


def _w(rng, N, K):
    return (rng.standard_normal((N, K)) * 0.02).astype(np.float16)


@pytest.mark.parametrize("M,K,group", [(300, 768, 128), (77, 512, 256), (1, 256, 0), (130, 1536, 384), (2100, 3072, 128)])
def test_quantize_act_operand_layout(B, orc, M, K, group):
    rng = np.random.default_rng(M + K + group)
    X = _x(rng, M, K)
    A = B.quantize_act(dev(X), ASYM, group, layout=MFMA)
    want = orc.quantize_act(X, ASYM, group)
    assert np.array_equal(act_to_canonical(host(A.q), ASYM), want["q"])
    assert np.array_equal(host(A.scale).view(np.uint32), want["s"].view(np.uint32))
    assert np.array_equal(host(A.zero).view(np.uint32), want["z"].view(np.uint32))
    assert np.array_equal(host(A.gsum), want["gsum"])
    G = K if group == 0 else group
    codes = orc.unpack(want["q"], ASYM).astype(np.int64).reshape(M, K // G, G)
    even = codes[:, :, 0::2].sum(axis=2)                           # [M, ng]
    assert np.array_equal(host(A.osum).astype(np.int64), 128 * even.T)   # group-major, pre-multiplied


@pytest.mark.parametrize("N,K,group", [(520, 768, 128), (64, 512, 256), (8, 256, 0), (1032, 3072, 128)])
def test_quantize_weight_operand_layout(B, orc, N, K, group):
    rng = np.random.default_rng(N + K + group)
    W = _w(rng, N, K)
    Q = B.quantize_weight(dev(W), ASYM, group, layout=MFMA)
    want = orc.quantize_weight(W, ASYM, group)
    assert np.array_equal(wgt_to_canonical(host(Q.q), ASYM), want["q"])
    for k in ("s", "z", "c"):
        assert np.array_equal(qweight_host(Q)[k].view(np.uint32), want[k].view(np.uint32)), k
    G = K if group == 0 else group
    ng = K // G
    codes = orc.unpack(want["q"], ASYM).astype(np.int64).reshape(N, ng, G)
    odd = codes[:, :, 1::2].sum(axis=2)
    es = host(Q.esum)
    assert es.shape == (N, ng + 1) and np.array_equal(es[:, :ng].astype(np.int64), odd)
    kw = es[:, ng].copy().view(np.float32).astype(np.float64)
    ref = 8.0 * (want["s"].reshape(N, ng).astype(np.float64) * odd).sum(axis=1)
    np.testing.assert_allclose(kw, ref, rtol=1e-6, atol=1e-6 * np.abs(ref).max())


def _layer(B, orc, rng, M, N, K, group, outliers=4):
    X, W = _x(rng, M, K, outliers), _w(rng, N, K)
    A = B.quantize_act(dev(X), ASYM, group, layout=MFMA)
    Q = B.quantize_weight(dev(W), ASYM, group, layout=MFMA)
    return A, Q, qact_host(A), qweight_host(Q)


@pytest.mark.parametrize("M,N,K,group", [(301, 520, 384, 128), (128, 128, 256, 0), (1, 8, 256, 128), (700, 1032, 1024, 256),
                                         (257, 264, 3072, 128), (140, 200, 1536, 512)])
def test_gemm_i32_exact(B, orc, M, N, K, group):
    rng = np.random.default_rng(M * 7 + N + K + group)
    A, Q, a, w = _layer(B, orc, rng, M, N, K, group)
    assert B.pick_schedule(A, Q) == "group_128x128"
    got = host(B.gemm_i32(A, Q))
    assert np.array_equal(got, orc.gemm_i32(a["q"], w["q"], ASYM, group))


def test_extreme_codes(B):
    """All-15 operands at K = 3072 in 24 groups: the largest group sums (225 * 128) and token / channel sums."""
    M, N, K, G = 130, 136, 3072, 128
    ng = K // G
    # canonical 0xFF -> activations 0xFF ^ 0x80 = 0x7F; weights: nibbles swapped, high nibble u - 8: 0x7F as well
    Aq = torch.full((M, K // 2), 0x7F, dtype=torch.uint8, device="cuda")
    Wq = torch.full((N, K // 2), 0x7F, dtype=torch.uint8, device="cuda")
    one = torch.ones(max(M, N) * ng, dtype=torch.float32, device="cuda")
    ra = torch.full((M, ng), 15 * G, dtype=torch.int32, device="cuda")
    ae = torch.full((ng, M), 128 * 15 * (G // 2), dtype=torch.int32, device="cuda")
    wo = torch.full((N, ng + 1), 15 * (G // 2), dtype=torch.int32, device="cuda")
    A = B.QAct(Aq, one[:M], one[:M], ra, M, K, K // 2, G, ASYM, 0, MFMA, ae)
    Q = B.QWeight(Wq, one[:N * ng].reshape(N, ng), one[:N * ng].reshape(N, ng), None, one[:N], N, K, G, ASYM,
                  MFMA, wo)
    assert (host(B.gemm_i32(A, Q)) == 225 * G).all()


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("M,N,K,group,bias", [(419, 776, 768, 128, True), (300, 264, 3072, 128, True), (150, 256, 512, 256, False),
                                              (1300, 136, 256, 0, True)])
def test_linear_fp16(B, orc, act, M, N, K, group, bias):
    rng = np.random.default_rng(M + N + K + group + act)
    A, Q, a, w = _layer(B, orc, rng, M, N, K, group)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16) if bias else None
    want = orc.linear(a, w, ASYM, group, b, act)
    got = host(B.linear(A, Q, None if b is None else dev(b), act))
    ok, ratio = f16_close_budget(got, want["out"], asym_budget(orc, a, w, group))
    assert ok, ratio
    # against the float64 evaluation of the dequantized operands: no further from it than the oracle's fp32 order is
    truth = orc.truth64(a, w, ASYM, b, act)
    e_gpu = np.sqrt(np.mean((got.astype(np.float64) - truth) ** 2))
    e_orc = np.sqrt(np.mean((want["out"].astype(np.float64) - truth) ** 2))
    same, steps = f16_steps(got, want["out"])
    print(f"M={M} N={N} K={K} G={group} act={act}: identical {same:.4f}, max steps {steps}, rms error vs float64: gpu {e_gpu:.3e} oracle {e_orc:.3e}")
    assert e_gpu <= 1.5 * e_orc + 1e-7


@pytest.mark.parametrize("group,K", [(128, 768), (256, 1024)])
def test_many_tiles_and_the_canonical_kernel(B, orc, group, K):
    """More tiles than resident workgroups, ragged M and N; sampled rows against the oracle, and the whole output
    against the same kernel on canonical codes (the two differ only in fp32 rounding order)."""
    rng = np.random.default_rng(600 + group)
    M, N = 128 * 11 + 37, 128 * 50 + 24
    X, W = _x(rng, M, K), _w(rng, N, K)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16)
    A = B.quantize_act(dev(X), ASYM, group, layout=MFMA)
    Q = B.quantize_weight(dev(W), ASYM, group, layout=MFMA)
    Ac, Qc = B.quantize_act(dev(X), ASYM, group), B.quantize_weight(dev(W), ASYM, group)
    rows = np.sort(np.concatenate([[0, M - 1], rng.choice(M, 30, replace=False)]))
    a, w = qact_host(A), qweight_host(Q)
    a = {k: (None if v is None else v[rows]) for k, v in a.items()}
    assert np.array_equal(host(B.gemm_i32(A, Q))[:, rows], orc.gemm_i32(a["q"], w["q"], ASYM, group))
    assert torch.equal(B.gemm_i32(A, Q), B.gemm_i32(Ac, Qc))
    for act in (0, 1):
        got = host(B.linear(A, Q, dev(b), act))
        want = orc.linear(a, w, ASYM, group, b, act)
        budget = asym_budget(orc, a, w, group)
        ok, ratio = f16_close_budget(got[rows], want["out"], budget)
        assert ok, ratio
        canon = host(B.linear(Ac, Qc, dev(b), act))                 # the oracle's operation order, every token
        assert np.array_equal(canon[rows].view(np.uint16), want["out"].view(np.uint16)) or act == 1
        worst = np.abs(got.astype(np.float64) - canon.astype(np.float64)).max(axis=1)    # per token, against the sampled budget
        assert worst.max() <= 1e-2 * np.abs(canon.astype(np.float64)).max() + 4 * budget.max(), float(worst.max())
