"""GPU-vs-oracle parity, element by element, through the C ABI (ctypes binding).

Bars: packed codes, scales, zero points, code sums and int32 accumulators are compared
bit for bit.  fp16 outputs must satisfy |gpu - oracle| <= 1e-2*|oracle| + 1e-3*rms(oracle)
(the stated 1e-2 relative target with an absolute floor); where the epilogue has no GELU
both sides perform the same separately rounded fp32 operations, so those outputs are
additionally required to be identical.  Requantized codes behind a GELU may differ by one
step only where the oracle's pre-rounding value sits within 1e-3 of a half-integer (the
device GELU and the oracle's differ by a few 1e-6 relative).
"""
import numpy as np
import pytest
import torch

from tests.gpu_util import GELU_SAME, assert_f16, dev, f16_close, has_gpu, host, qact_host, qweight_host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]

SYM, ASYM = 0, 1


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


def _rand_x(rng, M, K, outliers=0):
    x = rng.standard_normal((M, K)).astype(np.float32)
    if outliers:
        x[:, rng.choice(K, outliers, replace=False)] *= 20
    return x.astype(np.float16)


def _rand_w(rng, N, K):
    return (rng.standard_normal((N, K)) * 0.02).astype(np.float16)


# ------------------------------------------------------------------ step a1
@pytest.mark.parametrize("mode", [SYM, ASYM])
@pytest.mark.parametrize("M,K,group", [(1, 32, 0), (5, 96, 32), (130, 768, 128), (67, 1024, 128),
                                       (33, 4096, 128), (9, 3072, 0), (3, 8192, 1024), (2, 16384, 128)])
def test_quantize_act_bit_exact(B, orc, mode, M, K, group):
    rng = np.random.default_rng(100 + M + K + mode)
    X = _rand_x(rng, M, K, outliers=4 if K >= 96 else 0)
    X[0, :] = 0                                         # a constant (all-zero) token
    if M > 2:
        X[2, :] = X[2, 0]                               # a constant non-zero token
    want = orc.quantize_act(X, mode, group)
    A = B.quantize_act(dev(X), mode, group)
    if mode == SYM:                                     # code sums are optional for SYM: ask for them
        A.gsum = torch.empty((M, want["gsum"].shape[1]), dtype=torch.int32, device="cuda")
        A = B.quantize_act(dev(X), mode, group, out=A)
    torch.cuda.synchronize()
    assert np.array_equal(host(A.q), want["q"])
    assert np.array_equal(host(A.scale).view(np.uint32), want["s"].view(np.uint32))
    if mode == ASYM:
        assert np.array_equal(host(A.zero).view(np.uint32), want["z"].view(np.uint32))
    assert np.array_equal(host(A.gsum), want["gsum"])


def test_quantize_act_row_stride(B, orc):
    rng = np.random.default_rng(7)
    wide = _rand_x(rng, 40, 512)
    Xd = dev(wide)[:, 128:384]                           # a column slice: ldx = 512, K = 256
    A = B.quantize_act(Xd, SYM)
    want = orc.quantize_act(np.ascontiguousarray(wide[:, 128:384]), SYM)
    assert np.array_equal(host(A.q), want["q"]) and np.array_equal(host(A.scale), want["s"])


def test_quantize_act_extreme_values(B, orc):
    """fp16 subnormals, the largest finite values and exact ties keep CPU and GPU identical."""
    rows = []
    rows.append(np.full(64, 2.0 ** -24))                 # smallest subnormal everywhere
    r = np.zeros(64); r[0] = 65504; r[1] = -65504; r[2] = 2.0 ** -24; r[3] = 1.0; rows.append(r)
    r = np.zeros(64); r[0] = 7; r[1:15] = np.arange(0.5, 7.5, 0.5); rows.append(r)          # ties at inv = 1
    r = np.zeros(64); r[0] = 2.0 ** -23; r[1] = 2.0 ** -24; rows.append(r)                   # tie 3.5
    r = np.linspace(-3, 3, 64); rows.append(r)
    X = np.array(rows, np.float64).astype(np.float16)
    for mode in (SYM, ASYM):
        want = orc.quantize_act(X, mode)
        A = B.quantize_act(dev(X), mode)
        assert np.array_equal(host(A.q), want["q"]), mode
        assert np.array_equal(host(A.scale).view(np.uint32), want["s"].view(np.uint32))


# ------------------------------------------------------------------ step a0
@pytest.mark.parametrize("mode,group", [(SYM, 0), (SYM, 128), (ASYM, 0), (ASYM, 128), (ASYM, 256)])
def test_quantize_weight_bit_exact(B, orc, mode, group):
    rng = np.random.default_rng(200 + mode + group)
    W = _rand_w(rng, 72, 768)
    W[3, :] = 0
    want = orc.quantize_weight(W, mode, group)
    Q = B.quantize_weight(dev(W), mode, group)
    got = qweight_host(Q)
    assert np.array_equal(got["q"], want["q"])
    assert np.array_equal(got["s"].view(np.uint32), want["s"].view(np.uint32))
    assert np.array_equal(got["gsum"], want["gsum"])
    if mode == ASYM:
        assert np.array_equal(got["z"].view(np.uint32), want["z"].view(np.uint32))
    assert np.array_equal(got["c"].view(np.uint32), want["c"].view(np.uint32))


# ------------------------------------------------------------------ step a2
def _operands(B, orc, rng, M, N, K, mode, group, outliers=0):
    X, W = _rand_x(rng, M, K, outliers), _rand_w(rng, N, K)
    A = B.quantize_act(dev(X), mode, group)
    Q = B.quantize_weight(dev(W), mode, group)
    return X, W, A, Q


def _schedules(B, grouped, K=128):
    """Schedule numbers to exercise: every one that supports the layer (the pipelined kernel
    takes symmetric per-channel layers with K % 128 == 0, the split-K kernel K % 64 == 0)."""
    out = []
    for i, name in enumerate(B.schedule_names()):
        if name.startswith("olay") or name.startswith("fp6"):   # read their own operand layouts (tests/test_gpu_olay.py, test_gpu_fp6.py)
            continue
        if name.startswith("group") and (not grouped or K % 128 or K < 256):
            continue
        if name.startswith("small") and (grouped or K % 64 or K > 4096):   # symmetric per-channel, K % 64 == 0
            continue
        if name.startswith("pipe") and (grouped or K % 128):
            continue
        out.append(i + 1)
    return out


@pytest.mark.parametrize("mode,group", [(SYM, 0), (SYM, 128), (ASYM, 128), (ASYM, 0)])
def test_gemm_i32_bit_exact_every_schedule(B, orc, mode, group):
    """Several tiles in both directions with ragged tails in M, N and (ungrouped) K."""
    rng = np.random.default_rng(300 + mode + group)
    M, N = 301, 520
    grouped = not (mode == SYM and group == 0)
    for K in ((416, 384) if not grouped else (384,)):
        X, W, A, Q = _operands(B, orc, rng, M, N, K, mode, group)
        want = orc.gemm_i32(host(A.q), host(Q.q), mode, group)
        scheds = _schedules(B, grouped, K)
        assert len(scheds) >= 3                                   # the generic tiles, plus what the layer allows
        for sch in scheds:
            got = host(B.gemm_i32(A, Q, schedule=sch))
            assert got.shape == want.shape
            assert np.array_equal(got, want), f"K={K} schedule {sch} ({B.schedule_names()[sch - 1]})"


def test_gemm_i32_extreme_codes(B, orc):
    """All-(-8) and all-(+7) operands at K = 4096: the largest magnitudes the accumulators see."""
    K, M, N = 4096, 64, 64
    for ca, cw, val in ((0x88, 0x88, 64 * K), (0x77, 0x77, 49 * K), (0x77, 0x88, -56 * K)):
        Aq = torch.full((M, K // 2), ca, dtype=torch.uint8, device="cuda")
        Wq = torch.full((N, K // 2), cw, dtype=torch.uint8, device="cuda")
        one = torch.ones(max(M, N), dtype=torch.float32, device="cuda")
        A = B.QAct(Aq, one, None, None, M, K, K // 2, 0, SYM)
        Q = B.QWeight(Wq, one.reshape(-1, 1), None, None, None, N, K, 0, SYM)
        for sch in _schedules(B, False, K):                        # every kernel family that reads canonical symmetric codes
            P = host(B.gemm_i32(A, Q, schedule=sch))
            assert (P == val).all()
    Aq = torch.full((M, K // 2), 0xFF, dtype=torch.uint8, device="cuda")
    one = torch.ones(max(M, N), dtype=torch.float32, device="cuda")
    zi = torch.zeros((M, 1), dtype=torch.int32, device="cuda")
    A = B.QAct(Aq, one, one, zi, M, K, K // 2, 0, ASYM)
    Q = B.QWeight(Aq, one.reshape(-1, 1), one.reshape(-1, 1), None, one, N, K, 0, ASYM)
    for sch in _schedules(B, True, K):                              # ... and unsigned ones
        assert (host(B.gemm_i32(A, Q, schedule=sch)) == 225 * K).all(), sch


# ------------------------------------------------------------------ steps a2+a3 fused
def _oracle_layer(orc, A, Q, mode, group, bias, act, **kw):
    return orc.linear(qact_host(A), qweight_host(Q), mode, group, bias, act, **kw)


@pytest.mark.parametrize("mode,group,act", [(SYM, 0, 0), (SYM, 0, 1), (SYM, 128, 0), (ASYM, 128, 0),
                                            (ASYM, 128, 1), (ASYM, 0, 0)])
def test_linear_fp16_every_schedule(B, orc, mode, group, act):
    rng = np.random.default_rng(400 + 7 * mode + group + act)
    M, N, K = 291, 328, 384
    X, W, A, Q = _operands(B, orc, rng, M, N, K, mode, group, outliers=4 if mode == ASYM else 0)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    want = _oracle_layer(orc, A, Q, mode, group, bias, act)
    grouped = not (mode == SYM and group == 0)
    for sch in _schedules(B, grouped, K):
        got = host(B.linear(A, Q, dev(bias), act, schedule=sch))
        ok, ratio = f16_close(got, want["out"])
        assert ok, f"schedule {sch}: tolerance ratio {ratio}"
        assert_f16(got, want["out"], 1.0 if act == 0 else GELU_SAME, f"schedule {sch}")


def test_linear_without_bias(B, orc):
    rng = np.random.default_rng(41)
    X, W, A, Q = _operands(B, orc, rng, 64, 96, 256, SYM, 0)
    want = _oracle_layer(orc, A, Q, SYM, 0, None, 0)
    got = host(B.linear(A, Q, None, 0))
    assert np.array_equal(got.view(np.uint16), want["out"].view(np.uint16))


def test_dequant_epilogue_equals_fused_path(B, orc):
    """The stand-alone epilogue on exported accumulators reproduces the fused kernel bit for bit,
    for fp16 stores and for requantized outputs."""
    rng = np.random.default_rng(42)
    for mode, group in ((SYM, 0), (ASYM, 128)):
        M, N, K = 150, 256, 384
        X, W, A, Q = _operands(B, orc, rng, M, N, K, mode, group)
        bias = dev((rng.standard_normal(N) * 0.01).astype(np.float16))
        acc = B.gemm_i32(A, Q)
        for act in (0, 1):
            fused = host(B.linear(A, Q, bias, act))
            alone = host(B.dequant_epilogue(acc, A, Q, bias, act))
            assert np.array_equal(fused.view(np.uint16), alone.view(np.uint16)), (mode, act)
            for rmode in (SYM, ASYM):
                f = B.linear(A, Q, bias, act, requant=True, requant_mode=rmode, requant_group=128)
                a = B.dequant_epilogue(acc, A, Q, bias, act, requant=True, requant_mode=rmode, requant_group=128)
                assert np.array_equal(host(f.q), host(a.q)), (mode, act, rmode)
                assert np.array_equal(host(f.scale), host(a.scale))
                if rmode == ASYM:
                    assert np.array_equal(host(f.zero), host(a.zero))
                    assert np.array_equal(host(f.gsum), host(a.gsum))


def _requant_codes_agree(orc, got_q, want, y_f32, rmode, tau=1e-3):
    """Codes equal, except +-1 where the oracle's scaled value is within tau of a half-integer."""
    gq = orc.unpack(got_q, rmode).astype(np.int32)
    wq = orc.unpack(want["q"], rmode).astype(np.int32)
    diff = gq != wq
    if not diff.any():
        return 0
    s = want["s"].astype(np.float64)[:, None]
    z = want["z"].astype(np.float64)[:, None] if rmode == ASYM else 0.0
    t = (y_f32.astype(np.float64) - z) / s
    frac = np.abs(t - np.floor(t) - 0.5)
    assert np.all(np.abs(gq - wq)[diff] == 1)
    assert np.all(frac[diff] < tau), float(frac[diff].max())
    return int(diff.sum())


@pytest.mark.parametrize("mode,group", [(SYM, 0), (ASYM, 128)])
@pytest.mark.parametrize("rmode", [SYM, ASYM])
def test_linear_requant(B, orc, mode, group, rmode):
    rng = np.random.default_rng(500 + mode + rmode)
    M, N, K = 140, 384, 256
    X, W, A, Q = _operands(B, orc, rng, M, N, K, mode, group)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    # no GELU: identical fp32 sequences on both sides -> identical codes and scales
    want = _oracle_layer(orc, A, Q, mode, group, bias, 0, requant=True, requant_mode=rmode, requant_group=128)
    got = B.linear(A, Q, dev(bias), 0, requant=True, requant_mode=rmode, requant_group=128)
    assert np.array_equal(host(got.q), want["q"])
    assert np.array_equal(host(got.scale).view(np.uint32), want["s"].view(np.uint32))
    if rmode == ASYM:
        assert np.array_equal(host(got.zero).view(np.uint32), want["z"].view(np.uint32))
        assert np.array_equal(host(got.gsum), want["gsum"])
    # GELU: the device evaluates the erf form to ~5e-6 relative (the oracle uses libm's erf in
    # double) -> scales agree to 2e-5, codes are equal off near-ties
    want = _oracle_layer(orc, A, Q, mode, group, bias, 1, requant=True, requant_mode=rmode, requant_group=128)
    got = B.linear(A, Q, dev(bias), 1, requant=True, requant_mode=rmode, requant_group=128)
    np.testing.assert_allclose(host(got.scale), want["s"], rtol=2e-5)
    nd = _requant_codes_agree(orc, host(got.q), want, want["y"], rmode)
    assert nd <= 0.002 * M * N


def test_fused_requant_many_column_tiles(B, orc):
    """Symmetric per-channel layers requantize inside the GEMM kernel: the 16 column tiles of a
    row panel exchange per-token maxima through a workspace of a few words per token."""
    rng = np.random.default_rng(51)
    M, N, K = 700, 4096, 256
    X, W, A, Q = _operands(B, orc, rng, M, N, K, SYM, 0)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    need = B.linear_workspace_bytes(A, Q)
    assert need < 8 * M                                           # not the M*N*4 bytes of the two-kernel path
    assert B.linear_workspace_bytes(A, Q, requant_mode=ASYM) == M * N * 4
    assert B.linear_workspace_bytes(A, Q, want_gsum=True) == M * N * 4
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    want = _oracle_layer(orc, A, Q, SYM, 0, bias, 0, requant=True, requant_mode=SYM)
    for _ in range(2):                                            # the workspace is re-zeroed by every call
        got = B.linear(A, Q, dev(bias), 0, requant=True, requant_mode=SYM, workspace=ws)
        torch.cuda.synchronize()
        assert B.fused_fault(ws, need) == 0
        assert np.array_equal(host(got.q), want["q"])
        assert np.array_equal(host(got.scale).view(np.uint32), want["s"].view(np.uint32))
    # an all-zero token keeps scale 1 and codes 0 through the fused path as well
    Xz = X.copy(); Xz[5, :] = 0
    Az = B.quantize_act(dev(Xz), SYM)
    gz = B.linear(Az, Q, None, 0, requant=True, requant_mode=SYM, workspace=ws)
    assert float(host(gz.scale)[5]) == 1.0 and not host(gz.q)[5].any()


def test_fused_requant_at_the_residency_limit(B, orc):
    """The pipelined kernel's fused requantize needs its whole grid resident: 512 tiles (two workgroups on each
    of 256 CUs) still fuse, one row panel more falls back to fp32 rows + row quantizer; both give the same bits."""
    rng = np.random.default_rng(52)
    N, K = 4096, 256
    W = _rand_w(rng, N, K)
    Q = B.quantize_weight(dev(W), SYM)
    res = {}
    for M in (4096, 4224):
        X = _rand_x(rng, M, K)
        A = B.quantize_act(dev(X), SYM)
        need = B.linear_workspace_bytes(A, Q)
        res[M] = need
        got = B.linear(A, Q, None, 0, requant=True, requant_mode=SYM)
        acc = B.gemm_i32(A, Q)
        alone = B.dequant_epilogue(acc, A, Q, None, 0, requant=True, requant_mode=SYM)
        assert torch.equal(got.q, alone.q) and torch.equal(got.scale.view(torch.int32), alone.scale.view(torch.int32)), M
        rows = np.array([0, 127, 128, M // 2 + 3, M - 1])
        a = qact_host(A)
        a = dict(q=a["q"][rows], s=a["s"][rows], z=a["z"][rows], gsum=None)
        want = orc.linear(a, qweight_host(Q), SYM, 0, None, 0, requant=True, requant_mode=SYM)
        assert np.array_equal(host(got.q)[rows], want["q"])
    assert res[4096] < 8 * 4096 and res[4224] == 4224 * N * 4
    assert B.fused_fault_check() is False


def test_linear_reads_a_column_slice_in_place(B, orc):
    """lda > K/2: the GEMM reads the last third of a wider packed matrix (as the chained stack does)."""
    rng = np.random.default_rng(43)
    M, h = 70, 256
    X = _rand_x(rng, M, 3 * h)
    A3 = B.quantize_act(dev(X), SYM)
    Wv = _rand_w(rng, 128, h)
    Q = B.quantize_weight(dev(Wv), SYM)
    view = B.QAct(A3.q, A3.scale, None, None, M, h, A3.lda, 0, SYM, q_offset_bytes=h)
    got = host(B.linear(view, Q))
    a = qact_host(A3)
    a["q"] = np.ascontiguousarray(a["q"][:, h:h + h // 2])
    want = orc.linear(a, qweight_host(Q), SYM)
    assert np.array_equal(got.view(np.uint16), want["out"].view(np.uint16))


def test_degenerate_and_tiny_shapes(B, orc):
    rng = np.random.default_rng(44)
    for M, N, K in ((1, 8, 32), (2, 40, 64), (31, 8, 160), (257, 24, 32)):
        X, W, A, Q = _operands(B, orc, rng, M, N, K, SYM, 0)
        want = _oracle_layer(orc, A, Q, SYM, 0, None, 0)
        for sch in (0, B.schedule_number("generic_64x64"), B.schedule_number("generic_32x32")):
            got = host(B.linear(A, Q, schedule=sch))
            assert np.array_equal(got.view(np.uint16), want["out"].view(np.uint16)), (M, N, K, sch)
    # M == 0: nothing is launched, nothing fails
    A0 = B.QAct(torch.empty((0, 16), dtype=torch.uint8, device="cuda"), torch.empty(0, device="cuda"), None, None,
                0, 32, 16, 0, SYM)
    out = B.linear(A0, Q)
    assert out.shape == (0, 24)
    # all-zero activations: scale 1, codes 0, output = bias
    Xz = np.zeros((16, 64), np.float16)
    Az = B.quantize_act(dev(Xz), SYM)
    Wz = B.quantize_weight(dev(_rand_w(rng, 32, 64)), SYM)
    bias = (rng.standard_normal(32) * 0.01).astype(np.float16)
    got = host(B.linear(Az, Wz, dev(bias)))
    assert np.array_equal(got, np.broadcast_to(bias, (16, 32)))


def test_errors_raise(B):
    X = torch.zeros((4, 48), dtype=torch.float16, device="cuda")
    with pytest.raises(B.W4A4Error):
        B.quantize_act(X, SYM)                            # K % 32 != 0


@pytest.mark.parametrize("mode,group,K", [(ASYM, 128, 768), (ASYM, 0, 512), (SYM, 128, 512), (ASYM, 256, 1024)])
def test_grouped_kernel_many_tiles(B, orc, mode, group, K):
    """The persistent kernel for grouped / asymmetric layers with more tiles than resident workgroups
    (every workgroup walks several tiles; the group tables in LDS are replaced between tiles), ragged M
    and N; sampled rows against the oracle, int32 planes and fp16 outputs."""
    sch = B.schedule_names().index("group_128x128") + 1
    rng = np.random.default_rng(500 + mode + group + K)
    M, N = 128 * 11 + 37, 128 * 50 + 24                            # 12 x 51 = 612 tiles
    X, W, A, Q = _operands(B, orc, rng, M, N, K, mode, group, outliers=4 if mode == ASYM else 0)
    bias = (rng.standard_normal(N) * 0.01).astype(np.float16)
    rows = np.sort(np.concatenate([[0, M - 1], rng.choice(M, 30, replace=False)]))
    a, w = qact_host(A), qweight_host(Q)
    a = {k: (None if v is None else v[rows]) for k, v in a.items()}
    for act in (0, 1):
        want = orc.linear(a, w, mode, group, bias, act)
        got = host(B.linear(A, Q, dev(bias), act, schedule=sch))[rows]
        ok, ratio = f16_close(got, want["out"])
        assert ok, f"act {act}: tolerance ratio {ratio}"
        if act == 0:
            assert np.array_equal(got.view(np.uint16), want["out"].view(np.uint16))
    P = host(B.gemm_i32(A, Q, schedule=sch))[:, rows]
    assert np.array_equal(P, orc.gemm_i32(a["q"], w["q"], mode, group))
    # the shape table picks this kernel for large grouped layers: same result without naming it
    auto = host(B.linear(A, Q, dev(bias), 0))[rows]
    assert np.array_equal(auto, host(B.linear(A, Q, dev(bias), 0, schedule=sch))[rows])


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("M,K,ldx", [(8193, 32, 32), (8192, 160, 192), (9001, 1024, 1024), (8195, 2048, 2056), (8200, 992, 1000)])
def test_quantize_act_many_short_rows(B, orc, layout, M, K, ldx):
    """Thousands of short symmetric rows (more waves than the chip holds at once): odd row counts, ragged chunk
    counts and strided rows, in both layouts; the whole matrix against the oracle."""
    from tests.gpu_util import act_to_canonical
    rng = np.random.default_rng(M + K)
    Xw = (rng.standard_normal((M, ldx)) * rng.uniform(0.1, 4.0, size=(M, 1))).astype(np.float32).astype(np.float16)
    Xw[5, :] = 0                                              # an all-zero token
    Xw[M - 1, :K] = np.float16(65504.0)                       # the last row, at the top of the fp16 range
    Xd = dev(Xw)
    A = B.quantize_act(Xd[:, :K], SYM, layout=layout)
    want = orc.quantize_act(np.ascontiguousarray(Xw[:, :K]), SYM)
    q = host(A.q)
    assert np.array_equal(act_to_canonical(q) if layout == 1 else q, want["q"])
    assert np.array_equal(host(A.scale).view(np.uint32), want["s"].view(np.uint32))
    if layout == 1:
        odd = orc.unpack(want["q"], 0).astype(np.int64)[:, 1::2].sum(axis=1)
        assert np.array_equal(host(A.osum).astype(np.int64), odd)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("M,K,ldx,group", [(8193, 640, 648, 128), (8195, 1280, 1280, 128), (4100, 2560, 2568, 128),
                                           (9001, 96, 104, 0), (8200, 992, 1000, 0), (8191, 384, 384, 0),
                                           (4097, 3072, 3072, 128)])
def test_quantize_act_many_rows_asymmetric(B, orc, layout, M, K, ldx, group):
    """Thousands of asymmetric rows, several tokens per wave: odd row counts, chunk counts that do not fill the lanes
    of a token, strided rows, K-groups of 128 and one group per row, in both layouts; every output against the
    oracle (codes, scales, minima, K-group code sums, and the operand layout's 128 x even-position sums)."""
    from tests.gpu_util import act_to_canonical
    if layout == 1 and K % 128:
        pytest.skip("the operand layout of unsigned codes takes K in multiples of 128")
    rng = np.random.default_rng(M + K + group)
    Xw = (rng.standard_normal((M, ldx)) * rng.uniform(0.1, 4.0, size=(M, 1)) + rng.uniform(-2.0, 2.0, size=(M, 1)))
    Xw = Xw.astype(np.float32).astype(np.float16)
    Xw[5, :] = 0                                              # an all-zero token
    Xw[6, :] = np.float16(-3.25)                              # a constant token
    Xw[M - 1, :K] = np.float16(65504.0)                       # the last row: top of the fp16 range ...
    Xw[M - 1, K - 1] = np.float16(-65504.0)                   # ... to its bottom, in the last chunk
    Xd = dev(Xw)
    A = B.quantize_act(Xd[:, :K], ASYM, group, layout=layout)
    want = orc.quantize_act(np.ascontiguousarray(Xw[:, :K]), ASYM, group)
    q = host(A.q)
    assert np.array_equal(act_to_canonical(q, ASYM) if layout == 1 else q, want["q"])
    assert np.array_equal(host(A.scale).view(np.uint32), want["s"].view(np.uint32))
    assert np.array_equal(host(A.zero).view(np.uint32), want["z"].view(np.uint32))
    assert np.array_equal(host(A.gsum), want["gsum"])
    if layout == 1:
        G = K if group == 0 else group
        even = orc.unpack(want["q"], ASYM).astype(np.int64).reshape(M, K // G, G)[:, :, 0::2].sum(axis=2)
        assert np.array_equal(host(A.osum).astype(np.int64), 128 * even.T)
