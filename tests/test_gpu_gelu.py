"""The device GELU against the erf form in float64, over the whole range the layer can see."""
import math

import numpy as np
import pytest
import torch

from tests.gpu_util import dev, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]


def test_device_gelu_accuracy():
    """Drive the epilogue with P = code, sa = 1, sw = 1/64 so that y = code/64 exactly, add an
    fp16 bias to sweep a fine grid, and compare gelu(y) with 0.5*y*(1+erf(y/sqrt 2))."""
    from paper_2301_12017_amd import binding as B
    from scipy.special import erf
    M, N = 64, 1024
    # accumulators hold integers -512..511 -> y = acc/64 in [-8, 8); bias adds a sub-grid offset
    acc = torch.arange(-512, 512, dtype=torch.int32, device="cuda").repeat(M, 1).reshape(1, M, N).contiguous()
    bias = (np.arange(M * 0 + N) % 7 - 3).astype(np.float16) * np.float16(1.0 / 512)
    one = torch.ones(M, dtype=torch.float32, device="cuda")
    sw = torch.full((N, 1), 1.0 / 64, dtype=torch.float32, device="cuda")
    A = B.QAct(torch.zeros((M, 16), dtype=torch.uint8, device="cuda"), one, None, None, M, 32, 16, 0, 0)
    W = B.QWeight(torch.zeros((N, 16), dtype=torch.uint8, device="cuda"), sw, None, None, None, N, 32, 0, 0)
    y32 = B.dequant_epilogue(acc, A, W, dev(bias), B.ACT_GELU, requant=True, requant_mode=B.SYM)
    # requantized output hides values; use the fp16 path for the check instead
    y16 = host(B.dequant_epilogue(acc, A, W, dev(bias), B.ACT_GELU)).astype(np.float64)
    x = (np.arange(-512, 512) / 64.0)[None, :] + bias.astype(np.float64)[None, :]
    want = 0.5 * x * (1 + erf(x / math.sqrt(2)))
    # the layer's last operation (relu - t * Phi(-t)) is fused with the conversion and rounded once
    # to fp16, so the reference is rounded once as well (the grid is full of near-ties: y itself sits
    # on half-way points of the fp16 grid wherever the bias offset is odd)
    want16 = np.broadcast_to(want, (M, N)).astype(np.float16).astype(np.float64)
    err = np.abs(y16 - want16)
    ulp = np.maximum(np.abs(want16) * 2.0 ** -10, 2.0 ** -24)
    assert np.all(err <= ulp), float(np.max(err / ulp))            # at most one fp16 step anywhere
    assert np.mean(err == 0) > 0.93                                # (degree-5 tail: relative error < 9e-5)
    assert y32.scale.shape == (M,)
