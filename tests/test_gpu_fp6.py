"""GPU parity of the FP6 path: symmetric INT4 codes stored as FP6 E2M3 numbers, the GEMM on the FP6 matrix
instruction with FP32 accumulation (Sec. 4.2: INT4 arithmetic at twice the INT8 rate).  Codes, scales and int32
sums must equal the oracle's bit for bit; fp16 outputs without GELU too (the epilogue follows the definition's
operation order), with GELU within one fp16 step; outputs requantized in the GEMM epilogue (Sec. 4.2: the next
layer's quantize fused behind bias-add / GELU) equal the oracle's codes and scales bit for bit without GELU."""
import numpy as np
import pytest
import torch

from tests.gpu_util import GELU_SAME, assert_f16, dev, fp6_plan, fp6_schedules, fp6_to_codes, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]
SYM, FP6 = 0, 2


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def orc():
    import oracle
    return oracle


def _x(rng, M, K, outliers=4):
    x = rng.standard_normal((M, K)).astype(np.float32)
    if outliers:
        x[:, rng.choice(K, outliers, replace=False)] *= 20.0
    return x.astype(np.float16)


def _w(rng, N, K):
    return (rng.standard_normal((N, K)) * 0.02).astype(np.float16)


def test_plan_matches_the_library(B):
    """Row lengths the layout is not offered for (the quantizer's lane plan has no entry), and unsigned codes, are refused."""
    X = torch.zeros((8, 1792), dtype=torch.float16, device="cuda")          # 1792 / 32 = 56 = 8 * 7: seven operands per lane
    assert fp6_plan(1792) is None
    with pytest.raises(RuntimeError):
        B.quantize_act(X, SYM, layout=FP6)
    with pytest.raises(RuntimeError):
        B.quantize_act(torch.zeros((8, 320), dtype=torch.float16, device="cuda"), SYM, layout=FP6)   # K % 256 != 0
    with pytest.raises(RuntimeError):
        B.quantize_act(torch.zeros((8, 512), dtype=torch.float16, device="cuda"), 1, layout=FP6)     # unsigned codes


@pytest.mark.parametrize("M,K,ldx", [(1, 256, 256), (77, 512, 520), (300, 768, 768), (8193, 1024, 1024), (130, 1280, 1288),
                                     (67, 1536, 1536), (515, 2048, 2048), (2100, 3072, 3072), (1030, 4096, 4104),
                                     (33, 8192, 8192), (9, 10240, 10240)])
def test_quantize_act_fp6_layout(B, orc, M, K, ldx):
    rng = np.random.default_rng(M + K)
    Xw = (rng.standard_normal((M, ldx)) * rng.uniform(0.1, 4.0, size=(M, 1))).astype(np.float32).astype(np.float16)
    Xw[0, :] = 0                                              # an all-zero token
    Xw[M - 1, :K] = np.float16(65504.0)                       # top of the fp16 range ...
    Xw[M - 1, K - 1] = np.float16(-65504.0)                   # ... and its bottom
    if M > 2:
        Xw[1, :K] = np.float16(6e-8)                          # subnormals only
    A = B.quantize_act(dev(Xw)[:, :K], SYM, layout=FP6)
    want = orc.quantize_act(np.ascontiguousarray(Xw[:, :K]), SYM)
    assert A.q.shape == ((M + 63) // 64 * 64, K // 4 * 3) and A.lda == K // 4 * 3
    assert np.array_equal(fp6_to_codes(host(A.q), K, M), orc.unpack(want["q"], SYM))
    assert np.array_equal(host(A.scale).view(np.uint32), want["s"].view(np.uint32))


@pytest.mark.parametrize("N,K", [(8, 256), (520, 768), (64, 1024), (1032, 3072), (136, 4096)])
def test_quantize_weight_fp6_layout(B, orc, N, K):
    rng = np.random.default_rng(N + K)
    W = _w(rng, N, K)
    W[0, :] = 0
    Q = B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    want = orc.quantize_weight(W, SYM, 0)
    assert np.array_equal(fp6_to_codes(host(Q.q), K, N, weight=True), orc.unpack(want["q"], SYM))
    assert np.array_equal(host(Q.scale).view(np.uint32), want["s"].view(np.uint32))
    assert np.array_equal(host(Q.gsum), want["gsum"])
    assert np.array_equal(host(Q.rowsum_deq).view(np.uint32), want["c"].view(np.uint32))


def _layer(B, orc, rng, M, N, K):
    X, W = _x(rng, M, K), _w(rng, N, K)
    A, Q = B.quantize_act(dev(X), SYM, layout=FP6), B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    return A, Q, orc.quantize_act(X, SYM), orc.quantize_weight(W, SYM, 0)


@pytest.mark.parametrize("M,N,K", [(128, 256, 512), (300, 520, 768), (77, 136, 1024), (1, 8, 512), (515, 1032, 1280), (260, 264, 4096)])
def test_gemm_i32_bit_exact(B, orc, M, N, K):
    rng = np.random.default_rng(M * 3 + N + K)
    A, Q, a, w = _layer(B, orc, rng, M, N, K)
    want = orc.gemm_i32(a["q"], w["q"], SYM, 0)
    scheds = fp6_schedules(B, K)
    assert len(scheds) == (4 if K >= 640 else 3)
    for sch in scheds:
        got = host(B.gemm_i32(A, Q, schedule=sch))
        assert np.array_equal(got, want), f"schedule {B.schedule_names()[sch - 1]}"
    assert B.pick_schedule(A, Q).startswith("fp6")


def test_gemm_i32_extreme_codes(B, orc):
    """Every code at +-7 over K = 4096: the largest sums the layout can produce, 49 * 4096 = 200704 < 2^24."""
    M, N, K = 160, 264, 4096
    X = np.full((M, K), 3.0, np.float16)
    X[::2, ::3] = -3.0
    W = np.full((N, K), 0.5, np.float16)
    W[1::3, 1::2] = -0.5
    A, Q = B.quantize_act(dev(X), SYM, layout=FP6), B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    a, w = orc.quantize_act(X, SYM), orc.quantize_weight(W, SYM, 0)
    want = orc.gemm_i32(a["q"], w["q"], SYM, 0)
    assert np.abs(want).max() == 49 * 4096
    for sch in fp6_schedules(B, K):
        assert np.array_equal(host(B.gemm_i32(A, Q, schedule=sch)), want)


@pytest.mark.parametrize("act,with_bias", [(0, False), (0, True), (1, True), (1, False)])
def test_linear_fp16(B, orc, act, with_bias):
    M, N, K = 389, 1032, 1024
    rng = np.random.default_rng(7 + act + 2 * with_bias)
    A, Q, a, w = _layer(B, orc, rng, M, N, K)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float16) if with_bias else None
    want = orc.linear(a, w, SYM, 0, bias, act)["out"]
    for sch in fp6_schedules(B, K):
        got = host(B.linear(A, Q, dev(bias) if with_bias else None, act, schedule=sch))
        assert_f16(got, want, GELU_SAME if act else 1.0, f"schedule {B.schedule_names()[sch - 1]}")


@pytest.mark.parametrize("K", [512, 1024, 3072])
def test_many_tiles_per_workgroup(B, orc, K):
    """More tiles than resident workgroups: the stream of half steps runs across tile boundaries, in every tile shape;
    sampled rows (first, last, around panel boundaries) against the oracle."""
    M, N = 6144 + 70, 3072 + 8
    rng = np.random.default_rng(K)
    X, W = _x(rng, M, K), _w(rng, N, K)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float16)
    A, Q = B.quantize_act(dev(X), SYM, layout=FP6), B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(126, 130), np.arange(190, 194), np.arange(3070, 3074),
                                     rng.choice(M, 24, replace=False), np.arange(M - 3, M)]))
    a, w = orc.quantize_act(X[rows], SYM), orc.quantize_weight(W, SYM, 0)
    want_i = orc.gemm_i32(a["q"], w["q"], SYM, 0)
    want = orc.linear(a, w, SYM, 0, bias, 0)["out"]
    for sch in fp6_schedules(B, K):
        assert np.array_equal(host(B.gemm_i32(A, Q, schedule=sch))[0][rows], want_i[0]), B.schedule_names()[sch - 1]
        got = host(B.linear(A, Q, dev(bias), 0, schedule=sch))[rows]
        assert_f16(got, want, 1.0, B.schedule_names()[sch - 1])


def test_argument_errors(B):
    rng = np.random.default_rng(3)
    X, W = _x(rng, 64, 512), _w(rng, 64, 512)
    A = B.quantize_act(dev(X), SYM, layout=FP6)
    Qc = B.quantize_weight(dev(W), SYM, 0)                      # canonical weights against FP6 activations
    with pytest.raises(RuntimeError):
        B.linear(A, Qc, None, 0)
    Q = B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    with pytest.raises(RuntimeError):
        B.linear(A, Q, None, 0, schedule=B.schedule_number("olay_128x256"))   # a kernel of another layout
    X2, W2 = _x(rng, 64, 256), _w(rng, 64, 256)                 # the layout exists for K = 256, the GEMM wants K >= 512
    A2, Q2 = B.quantize_act(dev(X2), SYM, layout=FP6), B.quantize_weight(dev(W2), SYM, 0, layout=FP6)
    with pytest.raises(RuntimeError):
        B.linear(A2, Q2, None, 0)


@pytest.mark.parametrize("rmode,rlayout", [(SYM, 0), (1, 0), (SYM, 1)])
def test_requantized_output_from_fp6_operands(B, orc, rmode, rlayout):
    """A requantized output of a layer in the FP6 layout: the GEMM leaves fp32 rows (the definition's operation order) and the
    row quantizer packs them, in the canonical or the int8-MFMA operand layout: codes and scales equal the oracle's."""
    from tests.gpu_util import act_to_canonical
    M, N, K = 200, 512, 768
    rng = np.random.default_rng(11 + rmode + rlayout)
    A, Q, a, w = _layer(B, orc, rng, M, N, K)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    rg = 0 if rlayout == 1 else 128
    want = orc.linear(a, w, SYM, 0, bias, 0, requant=True, requant_mode=rmode, requant_group=rg)
    got = B.linear(A, Q, dev(bias), 0, requant=True, requant_mode=rmode, requant_group=rg, requant_layout=rlayout)
    q = host(got.q)
    assert np.array_equal(act_to_canonical(q) if rlayout == 1 else q, want["q"])
    assert np.array_equal(host(got.scale).view(np.uint32), want["s"].view(np.uint32))
    if rmode == 1:
        assert np.array_equal(host(got.zero).view(np.uint32), want["z"].view(np.uint32))


def _codes(want_q, N):
    """canonical packed nibbles (two's complement, low nibble first) -> int8 codes"""
    lo = (want_q & 15).astype(np.int8)
    hi = (want_q >> 4).astype(np.int8)
    c = np.empty(want_q.shape[:-1] + (N,), np.int8)
    c[..., 0::2] = np.where(lo > 7, lo - 16, lo)
    c[..., 1::2] = np.where(hi > 7, hi - 16, hi)
    return c


@pytest.mark.parametrize("M,N,K,bias", [(128, 256, 512, False), (200, 512, 768, True), (1000, 1024, 1024, True), (77, 768, 512, True),
                                        (2500, 3072, 1024, True), (1, 256, 512, True), (65, 256, 768, False), (64, 2560, 512, True),
                                        (129, 512, 10240, True), (300, 8192, 512, True)])
def test_fused_requantize_fp6(B, orc, M, N, K, bias):
    rng = np.random.default_rng(M + N + K)
    X, W = _x(rng, M, K), (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    A, Q = B.quantize_act(dev(X), SYM, layout=FP6), B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    a, w = orc.quantize_act(X, SYM), orc.quantize_weight(W, SYM, 0)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16) if bias else None
    want = orc.linear(a, w, SYM, 0, b, 0, requant=True, requant_mode=SYM, requant_group=0)
    got = B.linear(A, Q, dev(b) if bias else None, 0, requant=True, requant_mode=SYM, requant_group=0, requant_layout=FP6)
    torch.cuda.synchronize()
    assert B.fused_fault_check() == 0
    assert np.array_equal(host(got.scale).view(np.uint32), want["s"].view(np.uint32))
    codes = fp6_to_codes(host(got.q), N, M)
    assert np.array_equal(codes, _codes(want["q"], N))
    # the entry point without a workspace argument runs the same kernel on the library's static exchange area
    st = B.linear_static(A, Q, dev(b) if bias else None, 0, requant=True, requant_mode=SYM, requant_group=0, requant_layout=FP6)
    assert torch.equal(st.q, got.q) and torch.equal(st.scale, got.scale)


def test_chained_layers_and_column_slice(B, orc):
    """Two GEMMs in a row without an fp16 tensor between them: the requantized output of the first (GELU behind it) is the
    second's FP6 operand as it stands, once whole and once as its last third of columns read in place."""
    from paper_2301_12017_amd import workloads as WL
    M, K, N1, N2 = 300, 512, 1536, 256
    rng = np.random.default_rng(7)
    X, W1 = _x(rng, M, K), (rng.standard_normal((N1, K)) * 0.02).astype(np.float16)
    b1 = (rng.standard_normal(N1) * 0.01).astype(np.float16)
    A, Q1 = B.quantize_act(dev(X), SYM, layout=FP6), B.quantize_weight(dev(W1), SYM, 0, layout=FP6)
    H = B.linear(A, Q1, dev(b1), 0, requant=True, requant_layout=FP6)
    a, w1 = orc.quantize_act(X, SYM), orc.quantize_weight(W1, SYM, 0)
    h = orc.linear(a, w1, SYM, 0, b1, 0, requant=True, requant_mode=SYM, requant_group=0)
    assert np.array_equal(fp6_to_codes(host(H.q), N1, M), _codes(h["q"], N1))
    assert np.array_equal(host(H.scale).view(np.uint32), h["s"].view(np.uint32))
    # whole output as the next operand
    W2 = (rng.standard_normal((N2, N1)) * 0.02).astype(np.float16)
    Q2, w2 = B.quantize_weight(dev(W2), SYM, 0, layout=FP6), orc.quantize_weight(W2, SYM, 0)
    want = orc.gemm_i32(h["q"], w2["q"], SYM, 0)
    assert np.array_equal(host(B.gemm_i32(H, Q2)), want)
    # its last third of columns, in place
    third = N1 // 3
    W3 = (rng.standard_normal((N2, third)) * 0.02).astype(np.float16)
    Q3, w3 = B.quantize_weight(dev(W3), SYM, 0, layout=FP6), orc.quantize_weight(W3, SYM, 0)
    V = WL.v_slice(H, third)
    codes_v = _codes(h["q"], N1)[:, 2 * third:].astype(np.int64)
    want3 = codes_v @ _codes(w3["q"], third).astype(np.int64).T
    for sch in [i + 1 for i, n in enumerate(B.schedule_names()) if n.startswith("fp6") and n != "fp6_192x256"]:
        assert np.array_equal(host(B.gemm_i32(V, Q3, schedule=sch)).astype(np.int64).reshape(M, N2), want3)


def test_gelu_and_give_up(B, orc):
    """Behind a GELU the codes may differ from the oracle's by one step where the scaled value is next to a half-integer
    (the device's GELU is a polynomial); and a wait that cannot be satisfied ends with the fault flag, not a hang."""
    M, N, K = 640, 1024, 512
    rng = np.random.default_rng(9)
    X, W = _x(rng, M, K), (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    b = (rng.standard_normal(N) * 0.01).astype(np.float16)
    A, Q = B.quantize_act(dev(X), SYM, layout=FP6), B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    a, w = orc.quantize_act(X, SYM), orc.quantize_weight(W, SYM, 0)
    want = orc.linear(a, w, SYM, 0, b, 1, requant=True, requant_mode=SYM, requant_group=0)
    got = B.linear(A, Q, dev(b), 1, requant=True, requant_layout=FP6)
    codes, wc = fp6_to_codes(host(got.q), N, M).astype(np.int32), _codes(want["q"], N).astype(np.int32)
    np.testing.assert_allclose(host(got.scale), want["s"], rtol=2e-5)
    diff = np.abs(codes - wc)
    print("GELU requant: mismatching codes", int((diff != 0).sum()), "of", diff.size, flush=True)
    assert diff.max() <= 1 and (diff != 0).mean() <= 5e-5
    # the canonical output of the same layer (fp32 rows, then the row quantizer) holds the same codes
    ref = B.linear(A, Q, dev(b), 1, requant=True, requant_layout=0)
    assert np.array_equal(_codes(host(ref.q), N), codes)
    assert np.array_equal(host(ref.scale).view(np.uint32), host(got.scale).view(np.uint32))
    B.debug_fused_wait(64, 1)
    try:
        B.linear(A, Q, dev(b), 0, requant=True, requant_layout=FP6)
        torch.cuda.synchronize()
        assert B.fused_fault_check() is True
    finally:
        B.debug_fused_wait(0, 0)
    assert B.fused_fault_check() is False


@pytest.mark.parametrize("N,K,gelu", [(3072, 1024, False), (1024, 1024, False), (4096, 1024, True), (1024, 4096, False)])
def test_fused_requantize_fp6_at_full_size(B, N, K, gelu):
    """The four GEMMs of the chained workload at its 32768 tokens (several rounds of tiles per workgroup, every XCD's
    range of row panels): the fused kernel's FP6 codes and scales against the two-kernel path of the same operands
    (fp32 rows, then the row quantizer - the path compared with the oracle above), bit for bit, on both panels of every
    other row tile."""
    from paper_2301_12017_amd import synth
    M = 32768
    rng = np.random.default_rng(N + K)
    X = dev(synth.activations(M, K, 0, 5, 0))
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    b = dev((rng.standard_normal(N) * 0.01).astype(np.float16))
    A, Q = B.quantize_act(X, SYM, layout=FP6), B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    got = B.linear(A, Q, b, int(gelu), requant=True, requant_layout=FP6)
    assert B.pick_schedule(A, Q, requant=True, requant_layout=FP6) == "fp6_128x256"
    ref = B.linear(A, Q, b, int(gelu), requant=True, requant_layout=0)
    torch.cuda.synchronize()
    assert B.fused_fault_check() is False
    assert torch.equal(got.scale.view(torch.int32), ref.scale.view(torch.int32))
    panels = torch.arange(M // 64, device="cuda").view(-1, 2)[0::2].reshape(-1)          # both panels of every other 128-row tile
    q = got.q.view(M // 64, -1)[panels].cpu().numpy()
    rows = (panels[:, None] * 64 + torch.arange(64, device="cuda")[None, :]).reshape(-1)
    want = _codes(ref.q[rows].cpu().numpy(), N)
    for c0 in range(0, len(panels), 64):                                                   # 4096 rows at a time
        codes = fp6_to_codes(q[c0:c0 + 64], N, 64 * len(q[c0:c0 + 64]))
        assert np.array_equal(codes, want[64 * c0:64 * (c0 + 64)]), f"panels {c0} .. {c0 + 63} of the sample"


def test_fused_requantize_fp6_refusals(B):
    """What the fused FP6 output does not take is refused before anything is written."""
    rng = np.random.default_rng(2)
    X = dev(_x(rng, 128, 512))
    A = B.quantize_act(X, SYM, layout=FP6)
    Q = B.quantize_weight(dev(_w(rng, 384, 512)), SYM, 0, layout=FP6)                      # N not a multiple of 256
    with pytest.raises(RuntimeError):
        B.linear(A, Q, None, 0, requant=True, requant_layout=FP6)
    Q = B.quantize_weight(dev(_w(rng, 512, 512)), SYM, 0, layout=FP6)
    with pytest.raises(RuntimeError):                                                       # one range per token only
        B.linear(A, Q, None, 0, requant=True, requant_group=128, requant_layout=FP6)
    with pytest.raises(RuntimeError):                                                       # unsigned output codes
        B.linear(A, Q, None, 0, requant=True, requant_mode=1, requant_layout=FP6)
    Am = B.quantize_act(X, SYM, layout=1)
    Qm = B.quantize_weight(dev(_w(rng, 512, 512)), SYM, 0, layout=1)
    with pytest.raises(RuntimeError):                                                       # FP6 codes come from the FP6 kernel only
        B.linear(Am, Qm, None, 0, requant=True, requant_layout=FP6)


def test_calls_that_do_not_take_the_layout_refuse_it(B):
    rng = np.random.default_rng(5)
    W = _w(rng, 768, 768)
    Q = B.quantize_weight(dev(W), SYM, 0, layout=FP6)
    X = dev(_x(rng, 64, 768))
    with pytest.raises(RuntimeError):                          # one-launch small-token kernel: canonical weights only
        B.linear_f16act(X, Q, None, 0)


def test_headline_workload_at_full_size(B, orc):
    """Workload configs[2] (12288 tokens, BERT-large shapes) in the FP6 layout, in the launch configuration the bench
    times: codes and scales of sampled tokens, every weight code, and the fp16 outputs of 256 stratified rows per GEMM
    against the oracle (bit for bit without GELU; within one fp16 step behind it)."""
    from paper_2301_12017_amd import synth, workloads as WL
    rng = np.random.default_rng(33)
    for i, spec in enumerate(synth.config_linears(3)):
        layer = WL.make_layer(spec, 3, i, layout=FP6)
        X = WL.make_input(spec, 3, i)
        A = B.quantize_act(dev(X), SYM, layout=FP6)
        Y = B.linear(A, layer.W, layer.bias, layer.act)
        assert B.pick_schedule(A, layer.W).startswith("fp6")
        panels = (spec.M + 127) // 128
        rows = {0, spec.M - 1}
        order = rng.permutation(panels)
        k = 0
        while len(rows) < 256:
            rows.add(min(spec.M - 1, int(order[k % panels]) * 128 + int(rng.integers(128))))
            k += 1
        rows = np.array(sorted(rows))
        codes = fp6_to_codes(host(A.q), spec.K, spec.M)
        oa = orc.quantize_act(X[rows], SYM)
        assert np.array_equal(codes[rows], orc.unpack(oa["q"], SYM))
        assert np.array_equal(host(A.scale)[rows].view(np.uint32), oa["s"].view(np.uint32))
        ow = orc.quantize_weight(layer.host_W, SYM, 0)
        assert np.array_equal(fp6_to_codes(host(layer.W.q), spec.K, spec.N, weight=True), orc.unpack(ow["q"], SYM))
        want = orc.linear(oa, ow, SYM, 0, layer.host_b, 1 if spec.gelu else 0)["out"]
        assert_f16(host(Y)[rows], want, GELU_SAME if spec.gelu else 1.0, spec.name)
        del Y, A, layer
        torch.cuda.empty_cache()


@pytest.mark.parametrize("M,K,res", [(1, 256, False), (77, 768, True), (300, 1024, True), (130, 4096, False)])
def test_layernorm_quantize_into_the_fp6_layout(B, orc, M, K, res):
    """The fused producer writing the FP6 operand directly: the same codes, scales and fp16 copy as the call that writes
    canonical nibbles (one kernel, one arithmetic: bit for bit), which tests/test_gpu_layernorm.py holds against the oracle;
    and the result feeds the FP6 GEMM."""
    rng = np.random.default_rng(M + K)
    x = (rng.standard_normal((M, K)) * 1.7).astype(np.float32).astype(np.float16)
    r = rng.standard_normal((M, K)).astype(np.float16) if res else None
    g = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16)
    b = (0.1 * rng.standard_normal(K)).astype(np.float16)
    args = (dev(x), None if r is None else dev(r), dev(g), dev(b), 1e-5)
    A6, y6 = B.layernorm_quantize(*args, SYM, 0, layout=FP6)
    A0, y0 = B.layernorm_quantize(*args, SYM, 0, layout=0)
    assert torch.equal(y6, y0) and torch.equal(A6.scale, A0.scale)
    assert np.array_equal(fp6_to_codes(host(A6.q), K, M), orc.unpack(host(A0.q), 0).reshape(M, K))
    if K >= 512:
        W = _w(rng, 264, K)
        Q6, Q0 = B.quantize_weight(dev(W), SYM, 0, layout=FP6), B.quantize_weight(dev(W), SYM, 0)
        assert torch.equal(B.gemm_i32(A6, Q6), B.gemm_i32(A0, Q0))
    with pytest.raises(RuntimeError):                          # unsigned codes do not exist in this layout
        B.layernorm_quantize(*args, 1, 0, layout=FP6)
