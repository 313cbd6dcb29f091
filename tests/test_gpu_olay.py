"""GPU-vs-oracle parity for operands kept in the MFMA operand layout (w4a4_layout in w4a4.h).

The oracle knows one packing only (canonical two's-complement nibbles).  The operand layout is
a byte-wise bijection of it, so every comparison here first maps the device bytes back to
canonical bytes with the two functions below (bit operations only) and then asks for equality:
codes, scales, code sums and int32 accumulators bit for bit, fp16 outputs identical without
GELU and within the fp16 bar with it.
"""
import numpy as np
import pytest
import torch

from tests.gpu_util import (GELU_SAME, OLAY_SAME, act_to_canonical, assert_f16, dev, f16_close, has_gpu, host, olay_schedules,
                            wgt_to_canonical)

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]

SYM = 0
MFMA = 1


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


def _codes(orc, q_canonical):
    return orc.unpack(q_canonical, SYM).astype(np.int64)


def _rand_x(rng, M, K):
    return rng.standard_normal((M, K)).astype(np.float32).astype(np.float16)


def _rand_w(rng, N, K):
    return (rng.standard_normal((N, K)) * 0.02).astype(np.float16)


def _qhost(A, Q):
    a = dict(q=act_to_canonical(host(A.q)), s=host(A.scale), z=np.zeros(A.M, np.float32), gsum=None)
    w = dict(q=wgt_to_canonical(host(Q.q)), s=host(Q.scale), gsum=host(Q.gsum), c=host(Q.rowsum_deq))
    w["z"] = np.zeros_like(w["s"])
    return a, w


@pytest.mark.parametrize("M,K", [(1, 256), (130, 768), (67, 1024), (33, 4096), (3, 8192)])
def test_quantize_act_operand_layout(B, orc, M, K):
    rng = np.random.default_rng(900 + M + K)
    X = _rand_x(rng, M, K)
    X[0, :] = 0
    want = orc.quantize_act(X, SYM)
    A = B.quantize_act(dev(X), SYM, layout=MFMA)
    assert np.array_equal(act_to_canonical(host(A.q)), want["q"])
    assert np.array_equal(host(A.scale).view(np.uint32), want["s"].view(np.uint32))
    codes = _codes(orc, want["q"])
    assert np.array_equal(host(A.osum).astype(np.int64), codes[:, 1::2].sum(axis=1))


def test_quantize_weight_operand_layout(B, orc):
    rng = np.random.default_rng(901)
    W = _rand_w(rng, 72, 768)
    W[3, :] = 0
    want = orc.quantize_weight(W, SYM, 0)
    Q = B.quantize_weight(dev(W), SYM, 0, layout=MFMA)
    assert np.array_equal(wgt_to_canonical(host(Q.q)), want["q"])
    assert np.array_equal(host(Q.scale).view(np.uint32), want["s"].view(np.uint32))
    assert np.array_equal(host(Q.gsum), want["gsum"])
    codes = _codes(orc, want["q"])
    assert np.array_equal(host(Q.esum).astype(np.int64), codes[:, 0::2].sum(axis=1))


def test_layout_argument_errors(B):
    X = torch.zeros((4, 256), dtype=torch.float16, device="cuda")
    with pytest.raises(B.W4A4Error):                               # unsigned codes: the operand layout needs K % 128 == 0
        B.quantize_act(torch.zeros((4, 160), dtype=torch.float16, device="cuda"), 1, 0, layout=MFMA)
    A = B.quantize_act(X, SYM, layout=MFMA)
    Wc = B.quantize_weight(torch.zeros((8, 256), dtype=torch.float16, device="cuda"), SYM, 0)
    with pytest.raises(B.W4A4Error):
        B.gemm_i32(A, Wc)                                          # layouts of the two operands differ
    Wm = B.quantize_weight(torch.zeros((8, 256), dtype=torch.float16, device="cuda"), SYM, 0, layout=MFMA)
    with pytest.raises(B.W4A4Error):
        B.gemm_i32(A, Wm, schedule=B.schedule_number("pipe_128x256"))                              # that kernel reads canonical codes


def _olay_schedules(B, K):
    return olay_schedules(B, K)


@pytest.mark.parametrize("M,N,K", [(301, 520, 384), (128, 256, 256), (1, 8, 256), (700, 1032, 1024), (257, 264, 4096)])
def test_gemm_i32_bit_exact(B, orc, M, N, K):
    """Several tiles per workgroup, ragged tails in M and N, short and long K streams."""
    rng = np.random.default_rng(910 + M + N + K)
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    want = orc.gemm_i32(act_to_canonical(host(A.q)), wgt_to_canonical(host(Q.q)), SYM, 0)
    scheds = _olay_schedules(B, K)
    assert len(scheds) >= 2
    for sch in [0] + scheds:
        got = host(B.gemm_i32(A, Q, schedule=sch))
        assert got.shape == want.shape and np.array_equal(got, want), sch


def test_gemm_i32_extreme_codes(B):
    """All-(-8), all-(+7) and mixed operands at K = 4096: the largest magnitudes the accumulators
    and the code sums see."""
    K, M, N = 4096, 200, 264

    def enc_a(c):   # canonical byte of two equal codes -> activation operand byte
        return ((c & 0xF) | ((c & 0xF) << 4)) ^ 0x08

    def enc_w(c):
        return (((c + 8) & 0xF) | ((c & 0xF) << 4))

    one = torch.ones(max(M, N), dtype=torch.float32, device="cuda")
    for ca, cw in ((-8, -8), (7, 7), (7, -8), (-8, 7)):
        Aq = torch.full((M, K // 2), enc_a(ca), dtype=torch.uint8, device="cuda")
        Wq = torch.full((N, K // 2), enc_w(cw), dtype=torch.uint8, device="cuda")
        osum = torch.full((M,), ca * K // 2, dtype=torch.int32, device="cuda")
        esum = torch.full((N,), cw * K // 2, dtype=torch.int32, device="cuda")
        A = B.QAct(Aq, one, None, None, M, K, K // 2, 0, SYM, 0, MFMA, osum)
        Q = B.QWeight(Wq, one.reshape(-1, 1), None, None, None, N, K, 0, SYM, MFMA, esum)
        for sch in _olay_schedules(B, K):
            P = host(B.gemm_i32(A, Q, schedule=sch))
            assert (P == ca * cw * K).all(), (ca, cw, sch)


@pytest.mark.parametrize("act,with_bias", [(0, True), (1, True), (0, False), (1, False)])
def test_linear_fp16(B, orc, act, with_bias):
    rng = np.random.default_rng(920 + act + 2 * with_bias)
    M, N, K = 419, 776, 512
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16) if with_bias else None
    a, w = _qhost(A, Q)
    want = orc.linear(a, w, SYM, 0, bias, act)
    for sch in _olay_schedules(B, K):
        got = host(B.linear(A, Q, None if bias is None else dev(bias), act, schedule=sch))
        ok, ratio = f16_close(got, want["out"])
        assert ok, f"schedule {sch}: tolerance ratio {ratio}"
        assert_f16(got, want["out"], OLAY_SAME if act == 0 else GELU_SAME, f"schedule {sch}")


@pytest.mark.parametrize("K", [256, 768])
def test_many_tiles_per_workgroup(B, orc, K):
    """More tiles than resident workgroups (at most 3 x 256 CUs): every workgroup walks several tiles, so
    the K stream crosses tile boundaries (two K steps of the next tile are requested before the current
    one ends); sampled rows are checked against the oracle."""
    rng = np.random.default_rng(930 + K)
    M, N = 128 * 40, 256 * 30                                       # 1200 tiles of 128 x 256
    X = _rand_x(rng, M, K)
    A = B.quantize_act(dev(X), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    rows = np.sort(rng.choice(M, 48, replace=False))
    a, w = _qhost(A, Q)
    a = dict(q=a["q"][rows], s=a["s"][rows], z=a["z"][rows], gsum=None)
    want = orc.linear(a, w, SYM, 0, bias, 0)
    for sch in _olay_schedules(B, K):
        got = host(B.linear(A, Q, dev(bias), 0, schedule=sch))
        assert_f16(got[rows], want["out"], OLAY_SAME, f"schedule {sch}")
    # untouched rows would show up as the fill pattern: every output row was written
    P = host(B.gemm_i32(A, Q))
    wantP = orc.gemm_i32(a["q"], w["q"], SYM, 0)
    assert np.array_equal(P[0][rows], wantP[0])


def test_requantized_output_in_operand_layout(B, orc):
    """The requantizing epilogue can emit the next layer's operand layout directly."""
    rng = np.random.default_rng(940)
    M, N, K = 150, 512, 512
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    a, w = _qhost(A, Q)
    want = orc.linear(a, w, SYM, 0, bias, 0, requant=True, requant_mode=SYM)
    out = B.linear(A, Q, dev(bias), 0, requant=True, requant_mode=SYM, requant_layout=MFMA)
    assert out.layout == MFMA
    assert np.array_equal(act_to_canonical(host(out.q)), want["q"])
    assert np.array_equal(host(out.scale).view(np.uint32), want["s"].view(np.uint32))
    codes = _codes(orc, want["q"])
    assert np.array_equal(host(out.osum).reshape(M).astype(np.int64), codes[:, 1::2].sum(axis=1))


def _requant_compare(orc, want, out, gelu, M, N):
    """Scales and codes of a requantized output against the oracle's (canonical) ones."""
    gq = host(out.q)
    if out.layout == MFMA:
        gq = act_to_canonical(gq)
    gs = host(out.scale)
    if not gelu:
        assert np.array_equal(gs.view(np.uint32), want["s"].view(np.uint32))
        assert np.array_equal(gq, want["q"])
        return gq
    np.testing.assert_allclose(gs, want["s"], rtol=2e-5)
    gc, wc = orc.unpack(gq, SYM).astype(np.int32), orc.unpack(want["q"], SYM).astype(np.int32)
    diff = gc != wc
    t = want["y"].astype(np.float64) / want["s"].astype(np.float64)[:, None]
    frac = np.abs(t - np.floor(t) - 0.5)
    assert np.all(np.abs(gc - wc)[diff] == 1) and np.all(frac[diff] < 1e-4)
    print(f"GELU -> requantize {M}x{N}: {int(diff.sum())} of {diff.size} codes differ by one ({diff.mean():.2e}); "
          f"largest distance from the rounding boundary among them {float(frac[diff].max()) if diff.any() else 0.0:.2e}")
    assert diff.sum() <= max(2, 5e-5 * diff.size)
    return gq


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("M,N,K,group", [(300, 768, 512, 256), (1000, 3072, 256, 1024), (257, 1024, 1024, 0),
                                         (129, 288, 256, 0)])
def test_fused_requantize_operand_layout(B, orc, act, M, N, K, group):
    """One kernel: GEMM, dequantize, bias, (GELU), per-token requantize; codes leave in the operand
    layout with one odd-position sum per column slice.  Ragged M and (ungrouped) ragged N."""
    rng = np.random.default_rng(950 + M + N + act)
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    a, w = _qhost(A, Q)
    want = orc.linear(a, w, SYM, 0, bias, act, requant=True, requant_mode=SYM)
    need = B.linear_workspace_bytes(A, Q, requant_layout=MFMA, requant_group=group)
    assert need < M * N                                            # the fused path, not fp32 rows
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out = B.linear(A, Q, dev(bias), act, requant=True, requant_mode=SYM, requant_layout=MFMA, requant_group=group,
                   workspace=ws)
    torch.cuda.synchronize()
    assert B.fused_fault(ws, need) == 0
    gq = _requant_compare(orc, want, out, act == 1, M, N)
    codes = _codes(orc, gq)                                        # the sums must describe the codes that were written
    G = N if group == 0 else group
    sums = codes[:, 1::2].reshape(M, N // G, G // 2).sum(axis=2)
    assert np.array_equal(host(out.osum).reshape(M, -1).astype(np.int64), sums)
    # the same layer with canonical codes out
    need_c = B.linear_workspace_bytes(A, Q)
    ws_c = torch.empty(need_c, dtype=torch.uint8, device="cuda")
    out_c = B.linear(A, Q, dev(bias), act, requant=True, requant_mode=SYM, workspace=ws_c)
    torch.cuda.synchronize()
    assert need_c < M * N and B.fused_fault(ws_c, need_c) == 0 and out_c.layout == 0
    _requant_compare(orc, want, out_c, act == 1, M, N)


def test_fused_requantize_equals_dequant_epilogue(B, orc):
    """The stand-alone epilogue on exported accumulators reproduces the fused kernel's codes and scales."""
    rng = np.random.default_rng(960)
    M, N, K = 391, 1280, 768
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    bias = dev((rng.standard_normal(N) * 0.01).astype(np.float16))
    P = B.gemm_i32(A, Q)
    for act in (0, 1):
        fused = B.linear(A, Q, bias, act, requant=True, requant_mode=SYM, requant_layout=MFMA)
        alone = B.dequant_epilogue(P, A, Q, bias, act, requant=True, requant_mode=SYM)
        assert np.array_equal(act_to_canonical(host(fused.q)), host(alone.q)), act
        assert np.array_equal(host(fused.scale).view(np.uint32), host(alone.scale).view(np.uint32)), act


def test_chained_layers_in_operand_layout(B, orc):
    """Two encoder layers' worth of linears chained through requantized codes in the operand layout,
    the V third of the QKV output consumed in place; every GEMM teacher-forced against the oracle."""
    from paper_2301_12017_amd import synth, workloads as WL
    M, h, ffn = 700, 256, 1024
    X = synth.activations(M, h, 0, 5, 0)
    A = B.quantize_act(dev(X), SYM, layout=MFMA)
    for l in range(2):
        layer = WL.make_chain(1, h, ffn, M, 5, seed=l, layout=MFMA)[0]
        rec = []
        A = WL.run_chain(A, [layer], record=rec)
        for (_, name, a_in, out, lay) in rec:
            K = lay.spec.K
            off = a_in.q_offset_bytes
            qin = act_to_canonical(host(a_in.q))[:, off:off + K // 2]
            oin = dict(q=np.ascontiguousarray(qin), s=host(a_in.scale), z=np.zeros(M, np.float32), gsum=None)
            # the odd sums the consumer reads describe exactly these codes
            osum = host(a_in.osum).reshape(M, -1)[:, a_in.osum_index]
            assert np.array_equal(osum.astype(np.int64), _codes(orc, oin["q"])[:, 1::2].sum(axis=1)), (l, name)
            ow = orc.quantize_weight(lay.host_W, SYM)
            want = orc.linear(oin, ow, SYM, 0, lay.host_b, 1 if lay.spec.gelu else 0, requant=True)
            _requant_compare(orc, want, out, lay.spec.gelu, M, lay.spec.N)


def test_edge_shapes(B, orc):
    """Empty input, a single token, the narrowest output, the longest K the quantizers accept, and an
    activation matrix read as a column slice of a wider one (row stride > K/2, its own odd sums)."""
    rng = np.random.default_rng(970)
    Q = B.quantize_weight(dev(_rand_w(rng, 8, 256)), SYM, 0, layout=MFMA)
    A0 = B.QAct(torch.empty((0, 128), dtype=torch.uint8, device="cuda"), torch.empty(0, device="cuda"), None, None,
                0, 256, 128, 0, SYM, 0, MFMA, torch.empty(0, dtype=torch.int32, device="cuda"))
    assert B.linear(A0, Q).shape == (0, 8)                          # M == 0: a successful no-op
    for M, N, K in ((1, 8, 256), (3, 40, 16384)):
        A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
        Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
        a, w = _qhost(A, Q)
        assert np.array_equal(host(B.gemm_i32(A, Q))[0], orc.gemm_i32(a["q"], w["q"], SYM, 0)[0])
        want = orc.linear(a, w, SYM, 0, None, 0)
        assert_f16(host(B.linear(A, Q)), want["out"], 0.98, str((M, N, K)))    # (a handful of values: one near-tie allowed)
    # column slice: quantize a [M, 3K] matrix third by third into one packed buffer, multiply the middle third
    M, K, N = 200, 512, 136
    Xw = _rand_x(rng, M, 3 * K)
    wide = torch.empty((M, 3 * K // 2), dtype=torch.uint8, device="cuda")
    osum = torch.empty((M, 3), dtype=torch.int32, device="cuda")
    scales = []
    for t in range(3):
        At = B.quantize_act(dev(np.ascontiguousarray(Xw[:, t * K:(t + 1) * K])), SYM, layout=MFMA)
        wide[:, t * K // 2:(t + 1) * K // 2] = At.q
        osum[:, t] = At.osum
        scales.append(At.scale)
    Amid = B.QAct(wide, scales[1], None, None, M, K, 3 * K // 2, 0, SYM, q_offset_bytes=K // 2, layout=MFMA,
                  osum=osum, osum_index=1)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    want = orc.quantize_act(np.ascontiguousarray(Xw[:, K:2 * K]), SYM)
    w = _qhost(B.quantize_act(dev(np.ascontiguousarray(Xw[:, K:2 * K])), SYM, layout=MFMA), Q)[1]
    assert np.array_equal(host(B.gemm_i32(Amid, Q))[0], orc.gemm_i32(want["q"], w["q"], SYM, 0)[0])


def test_non_finite_inputs_do_not_fault(B):
    """NaN / Inf activations: results are unspecified, but every kernel must run to completion."""
    M, N, K = 300, 544, 512
    X = np.ones((M, K), np.float16)
    X[0, 0] = np.nan
    X[1, 5] = np.inf
    X[2, :] = -np.inf
    A = B.quantize_act(dev(X), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(np.ones((N, K), np.float16)), SYM, 0, layout=MFMA)
    Y = B.linear(A, Q, None, 1)
    Z = B.linear(A, Q, None, 1, requant=True, requant_layout=MFMA)
    torch.cuda.synchronize()
    assert Y.shape == (M, N) and Z.q.shape == (M, N // 2)
    assert np.isfinite(host(Y)[3:].astype(np.float32)).all()        # finite rows are unaffected by the others


def test_fused_requantize_widest_output(B, orc):
    """N = 8192 (32 column tiles exchange their maxima), sampled rows against the oracle."""
    rng = np.random.default_rng(980)
    M, N, K = 600, 8192, 256
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    need = B.linear_workspace_bytes(A, Q, requant_layout=MFMA, requant_group=2048)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out = B.linear(A, Q, None, 0, requant=True, requant_layout=MFMA, requant_group=2048, workspace=ws)
    torch.cuda.synchronize()
    assert need < M * N and B.fused_fault(ws, need) == 0
    rows = np.sort(rng.choice(M, 24, replace=False))
    a, w = _qhost(A, Q)
    a = dict(q=a["q"][rows], s=a["s"][rows], z=a["z"][rows], gsum=None)
    want = orc.linear(a, w, SYM, 0, None, 0, requant=True)
    assert np.array_equal(act_to_canonical(host(out.q))[rows], want["q"])
    assert np.array_equal(host(out.scale)[rows].view(np.uint32), want["s"].view(np.uint32))
    sums = _codes(orc, want["q"])[:, 1::2].reshape(len(rows), 4, 1024).sum(axis=2)
    assert np.array_equal(host(out.osum)[rows].astype(np.int64), sums)


def test_fused_requantize_gives_up_cleanly(B):
    """The bounded wait of the fused requantize, forced from the host: the kernels are told to wait for one
    more sibling tile than a row panel has and to poll a handful of times only.  Every workgroup then gives
    up, raises both fault words and exits normally; the next, ordinary call is unaffected."""
    rng = np.random.default_rng(985)
    M, N, K = 300, 768, 256
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=MFMA)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, 0, layout=MFMA)
    need = B.linear_workspace_bytes(A, Q, requant_layout=MFMA)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    assert B.fused_fault_check() is False
    good = B.linear(A, Q, None, 0, requant=True, requant_layout=MFMA, workspace=ws)
    torch.cuda.synchronize()
    assert B.fused_fault(ws, need) == 0 and B.fused_fault_check() is False
    B.debug_fused_wait(spin_limit=8, extra_arrivals=1)
    try:
        B.linear(A, Q, None, 0, requant=True, requant_layout=MFMA, workspace=ws)
        torch.cuda.synchronize()                                   # returns: nobody hangs
    finally:
        B.debug_fused_wait(0, 0)
    assert B.fused_fault(ws, need) != 0
    assert B.fused_fault_check() is True and B.fused_fault_check() is False    # reported once, then cleared
    again = B.linear(A, Q, None, 0, requant=True, requant_layout=MFMA, workspace=ws)
    torch.cuda.synchronize()
    assert B.fused_fault(ws, need) == 0 and B.fused_fault_check() is False
    assert torch.equal(again.q, good.q) and torch.equal(again.scale, good.scale) and torch.equal(again.osum, good.osum)


@pytest.mark.parametrize("N,K,gelu", [(3072, 1024, 0), (1024, 1024, 0), (4096, 1024, 1), (1024, 4096, 0)])
def test_fused_requantize_equals_two_kernel_path_at_full_size(B, N, K, gelu):
    """M = 32768 (the chained workload): the persistent kernel walks several rounds of tiles with panel waits on
    every XCD.  Its codes, scales and odd-position sums must equal, bit for bit and for EVERY token, those of
    the two-kernel path (fp32 rows, then the row quantizer), which involves no waiting."""
    M = 32768
    gen = torch.Generator(device="cuda").manual_seed(N + K)
    X = torch.randn((M, K), device="cuda", generator=gen).half()
    W = (torch.randn((N, K), device="cuda", generator=gen) * 0.02).half()
    bias = (torch.randn((N,), device="cuda", generator=gen) * 0.01).half()
    A = B.quantize_act(X, SYM, layout=MFMA)
    Q = B.quantize_weight(W, SYM, 0, layout=MFMA)
    need = B.linear_workspace_bytes(A, Q, requant_layout=MFMA)
    assert need < 8 * M
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    fused = B.linear(A, Q, bias, gelu, requant=True, requant_layout=MFMA, workspace=ws)
    torch.cuda.synchronize()
    assert B.fused_fault(ws, need) == 0
    other = B.schedule_number("olay_192x128")                      # a forced schedule other than the fused kernel's
    assert B.linear_workspace_bytes(A, Q, requant_layout=MFMA, schedule=other) == M * N * 4
    plain = B.linear(A, Q, bias, gelu, requant=True, requant_layout=MFMA, schedule=other)
    assert torch.equal(fused.q, plain.q)
    assert torch.equal(fused.scale.view(torch.int32), plain.scale.view(torch.int32))
    assert torch.equal(fused.osum.reshape(M), plain.osum.reshape(M))
    if N == 3072:                                                  # one sum per third: equal to sums over the code bytes
        sl = B.linear(A, Q, bias, gelu, requant=True, requant_layout=MFMA, requant_group=1024, workspace=ws)
        assert torch.equal(sl.q, plain.q)
        hi = (sl.q.to(torch.int32) >> 4)                            # odd positions: two's-complement high nibbles
        hi = torch.where(hi >= 8, hi - 16, hi).reshape(M, 3, 512).sum(dim=2)
        assert torch.equal(sl.osum.reshape(M, 3), hi.to(torch.int32))
    assert B.fused_fault_check() is False


@pytest.mark.parametrize("layout,M,N,K", [(MFMA, 2048, 512, 512), (0, 300, 256, 384)])
def test_kernel_timer_stamps_one_gemm(B, layout, M, N, K):
    """w4a4_time_next_gemm: the armed events bracket the GEMM kernel of the next call only, the
    arming is consumed by it, and the output does not depend on it."""
    rng = np.random.default_rng(31)
    A = B.quantize_act(dev(_rand_x(rng, M, K)), SYM, layout=layout)
    Q = B.quantize_weight(dev(_rand_w(rng, N, K)), SYM, layout=layout)
    plain = host(B.linear(A, Q, None, 0))
    t = B.KernelTimer()
    t.arm()
    timed = host(B.linear(A, Q, None, 0))                         # host() synchronizes
    ms = t.elapsed_ms()
    assert 0.0 < ms < 5.0
    assert np.array_equal(plain.view(np.uint16), timed.view(np.uint16))
    again = host(B.linear(A, Q, None, 0))                         # not armed any more
    assert t.elapsed_ms() == ms
    assert np.array_equal(plain.view(np.uint16), again.view(np.uint16))
