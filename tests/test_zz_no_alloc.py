"""w4a4_linear_static, the entry point for callers that cannot allocate: through the C ABI, against w4a4_linear
on the same operands, bit for bit, twice in a row with the second call on fewer tokens (the static exchange
area keeps the first call's contents until the second clears it)."""
import ctypes

import numpy as np
import pytest
import torch

from tests.gpu_util import has_gpu

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]

SYM, MFMA = 0, 1


def _operands(B, M, N, K, seed, layout):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    X = torch.randn((M, K), device="cuda", generator=gen).half()
    W = (torch.randn((N, K), device="cuda", generator=gen) * 0.02).half()
    bias = (torch.randn((N,), device="cuda", generator=gen) * 0.01).half()
    return B.quantize_act(X, SYM, layout=layout), B.quantize_weight(W, SYM, 0, layout=layout), bias


def _raw_static(B, A, Q, bias, act, out, layout, group):
    """The C call itself, with preallocated outputs: nothing is allocated between the two launches."""
    ep = B._Epilogue(bias.data_ptr(), act, 1, SYM, group, layout, 0)
    a, w = A.c(), Q.c()
    rc = B.lib().w4a4_linear_static(ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep), B._ptr(out[0]), B._ptr(out[1]),
                                    B._ptr(out[2]), B._ptr(out[3]), B._stream())
    assert rc == 0, B.status_string(rc)


@pytest.mark.parametrize("layout", [MFMA, 0])
def test_static_scratch_equals_workspace_path_twice_in_a_row(layout):
    from paper_2301_12017_amd import binding as B
    B.lib()
    N, K, group = 3072, 512, 1024 if layout == MFMA else 0
    big = _operands(B, 2500, N, K, 1, layout)                      # 20 row panels x 12 column tiles, ragged M
    small = _operands(B, 333, N, K, 2, layout)
    refs, outs = [], []
    for A, Q, bias in (big, small):
        refs.append(B.linear(A, Q, bias, 1, requant=True, requant_layout=layout, requant_group=group))
        outs.append(B._alloc_out(A, Q, True, SYM, group, layout))
    torch.cuda.synchronize()
    assert B.fused_fault_check() is False
    for (A, Q, bias), out in zip((big, small), outs):              # back to back on one stream, second call smaller
        _raw_static(B, A, Q, bias, 1, out, layout, group)
    torch.cuda.synchronize()
    assert B.fused_fault_check() is False
    for ref, out in zip(refs, outs):
        assert torch.equal(out[0], ref.q)
        assert torch.equal(out[1].view(torch.int32), ref.scale.view(torch.int32))
        if layout == MFMA:
            assert torch.equal(out[3], ref.osum)


def test_static_entry_point_without_requantize_and_its_limits():
    from paper_2301_12017_amd import binding as B
    B.lib()
    A, Q, bias = _operands(B, 300, 544, 512, 3, MFMA)
    assert torch.equal(B.linear_static(A, Q, bias, 1).view(torch.int16), B.linear(A, Q, bias, 1).view(torch.int16))
    # an asymmetric requantize cannot be fused: it would need fp32 rows, which this entry point has no room for
    with pytest.raises(B.W4A4Error) as e:
        B.linear_static(A, Q, bias, 0, requant=True, requant_mode=1)
    assert e.value.status == -3                                    # W4A4_ERR_WORKSPACE
    # more tokens than the static area holds: refused before anything is launched (fake pointers are never read)
    M = 65537
    big = B.QAct(A.q, A.scale, None, None, M, 512, 256, 0, SYM, 0, MFMA, A.osum)
    out = B._alloc_out(A, Q, True, SYM, 0, MFMA)
    ep = B._Epilogue(None, 0, 1, SYM, 0, MFMA, 0)
    a, w = big.c(), Q.c()
    rc = B.lib().w4a4_linear_static(ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep), B._ptr(out[0]), B._ptr(out[1]),
                                    None, B._ptr(out[3]), B._stream())
    assert rc == -3
