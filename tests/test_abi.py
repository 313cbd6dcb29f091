"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def b():
    from paper_2301_12017_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2301_12017_amd import build
        build.build(verbose=False)
    return binding


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "w4a4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(w[48]a[48]_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(b):
    names = _declared_symbols()
    assert {"w4a4_quantize_act", "w4a4_linear", "w4a4_dequant_epilogue", "w4a4_quantize_weight",
            "w4a4_gemm_i32", "w4a4_workspace_bytes"} <= set(names)
    L = ctypes.CDLL(b.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(b.EXPORTS)


def test_version_and_status_strings(b):
    assert "gfx950" in b.version()
    assert b.status_string(0) == "ok"
    for s in (-1, -2, -3, -4):
        assert b.status_string(s) not in ("ok", "unknown status")
    assert len(b.schedule_names()) == b.lib().w4a4_schedule_count() >= 1


def _act(b, M=4, K=64, lda=None, mode=0, group=0, ptr=0x1000, layout=0, osum=None, ldo=1):
    return b._Act(ptr, ptr, ptr, ptr, M, K, K // 2 if lda is None else lda, group, mode, layout, osum, ldo)


def _wt(b, N=8, K=64, mode=0, group=0, ptr=0x1000, layout=0, esum=None):
    return b._Weight(ptr, ptr, ptr, ptr, N, K, group, mode, layout, esum)


def test_argument_errors_are_reported_before_any_launch(b):
    """Pointers here are fake (never dereferenced): every call must fail in validation."""
    L = b.lib()
    ep = b._Epilogue(None, 0, 0, 0, 0, 0, 0)
    out = ctypes.c_void_p(0x2000)

    def lin(a, w, e=ep, o=out, ws=None, wsb=0, os_=None):
        return L.w4a4_linear(ctypes.byref(a), ctypes.byref(w), ctypes.byref(e), o, os_, None, None, ws, wsb, None)

    assert lin(_act(b, K=64), _wt(b, K=128)) == -1                    # K mismatch
    assert lin(_act(b, mode=0), _wt(b, mode=1)) == -1                 # mode mismatch
    assert lin(_act(b, K=48), _wt(b, K=48)) == -2                     # K % 32
    assert lin(_act(b), _wt(b, N=12)) == -2                           # N % 8
    assert lin(_act(b, lda=16), _wt(b)) == -1                         # lda < K/2
    assert lin(_act(b, lda=40), _wt(b)) == -2                         # lda % 16
    assert lin(_act(b, K=256), _wt(b, K=256, group=64)) == -2         # GEMM groups are multiples of 128
    assert lin(_act(b, K=256), _wt(b, K=256, group=96)) == -2         # group must divide K
    assert lin(_act(b, ptr=None), _wt(b)) == -1                       # null operand
    assert lin(_act(b), _wt(b), o=None) == -1                         # null output
    assert lin(_act(b, ptr=0x1004), _wt(b)) == -2                     # misaligned
    bad_act = b._Epilogue(None, 7, 0, 0, 0, 0, 0)
    assert lin(_act(b), _wt(b), e=bad_act) == -1
    rq = b._Epilogue(None, 0, 1, 0, 0, 0, 0)
    assert lin(_act(b), _wt(b, N=32), e=rq, os_=None) == -1           # requant needs out_scale
    assert lin(_act(b), _wt(b, N=32), e=rq, os_=out) == -3            # and a workspace
    assert lin(_act(b), _wt(b, N=8), e=rq, os_=out) == -2             # requant N % 32
    # asymmetric operands need zero points, code sums and the weight row sums
    a = _act(b, K=128, mode=1, group=128); a.gsum = None
    assert lin(a, _wt(b, K=128, mode=1, group=128)) == -1
    assert lin(_act(b, K=256, mode=1, group=0), _wt(b, K=256, mode=1, group=128)) == -1   # group mismatch
    # operands in the MFMA operand layout: both sides, symmetric, with their code sums, K % 128, K >= 256
    o = 0x3000
    assert lin(_act(b, K=256, layout=1, osum=o), _wt(b, K=256)) == -1                     # layouts differ
    assert lin(_act(b, K=256, layout=1), _wt(b, K=256, layout=1, esum=o)) == -1           # osum missing
    assert lin(_act(b, K=256, layout=1, osum=o), _wt(b, K=256, layout=1)) == -1           # esum missing
    assert lin(_act(b, K=256, layout=1, osum=o, ldo=0), _wt(b, K=256, layout=1, esum=o)) == -1
    assert lin(_act(b, K=128, layout=1, osum=o), _wt(b, K=128, layout=1, esum=o)) == -2   # K < 256
    assert lin(_act(b, K=256, layout=7, osum=o), _wt(b, K=256, layout=7, esum=o)) == -1
    rq_bad = b._Epilogue(None, 0, 1, 1, 0, 1, 0)                                          # ASYM codes in the operand layout
    assert lin(_act(b), _wt(b, N=32), e=rq_bad, os_=out) == -1
    # operands in the FP6 operand layout: symmetric, one scale per row, K % 256 == 0, K >= 512, lda >= 3K/4
    a6, w6 = _act(b, K=512, lda=384, layout=2), _wt(b, N=256, K=512, layout=2)
    assert lin(_act(b, K=512, lda=384, layout=2, mode=1), _wt(b, N=256, K=512, layout=2, mode=1)) == -1   # unsigned codes
    assert lin(_act(b, K=512, lda=256, layout=2), w6) == -1                               # lda < 3K/4
    assert lin(_act(b, K=320, lda=240, layout=2), _wt(b, N=256, K=320, layout=2)) == -2   # K % 128
    assert lin(_act(b, K=256, lda=192, layout=2), _wt(b, N=256, K=256, layout=2)) == -2   # K < 512
    assert lin(a6, _wt(b, N=256, K=512, layout=2, group=128)) == -2                       # K-groups
    # a requantized output in the FP6 layout: from FP6 operands only, symmetric, one range per token
    assert lin(_act(b), _wt(b, N=256), e=b._Epilogue(None, 0, 1, 0, 0, 2, 0), os_=out) == -2
    assert lin(a6, w6, e=b._Epilogue(None, 0, 1, 1, 0, 2, 0), os_=out) == -1
    assert lin(a6, w6, e=b._Epilogue(None, 0, 1, 0, 128, 2, 0), os_=out) == -2
    # M == 0 is a successful no-op
    assert lin(_act(b, M=0), _wt(b)) == 0
    assert L.w4a4_gemm_i32(ctypes.byref(_act(b)), ctypes.byref(_wt(b)), None, 0, None) == -1
    assert L.w4a4_gemm_i32(ctypes.byref(_act(b)), ctypes.byref(_wt(b)), out, 99, None) == -1


def test_quantize_argument_errors(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)
    assert L.w4a4_quantize_act(None, 4, 64, 64, 0, 0, p, p, None, None, 0, None, None) == -1
    assert L.w4a4_quantize_act(p, 4, 48, 48, 0, 0, p, p, None, None, 0, None, None) == -2
    assert L.w4a4_quantize_act(p, 4, 64, 32, 0, 0, p, p, None, None, 0, None, None) == -1      # ldx < K
    assert L.w4a4_quantize_act(p, 4, 64, 64, 1, 0, p, p, None, None, 0, None, None) == -1      # ASYM needs zero
    assert L.w4a4_quantize_act(p, 4, 64, 64, 0, 24, p, p, None, None, 0, None, None) == -2     # group % 32
    assert L.w4a4_quantize_act(p, 4, 32768, 32768, 0, 0, p, p, None, None, 0, None, None) == -2
    assert L.w4a4_quantize_act(p, 0, 64, 64, 0, 0, p, p, None, None, 0, None, None) == 0
    assert L.w4a4_quantize_act(p, 4, 64, 64, 0, 0, p, p, None, None, 1, None, None) == -1      # operand layout needs osum
    assert L.w4a4_quantize_act(p, 4, 64, 64, 1, 0, p, p, p, None, 1, p, None) == -2            # unsigned codes: whole K steps of 128
    assert L.w4a4_quantize_act(p, 4, 256, 256, 1, 64, p, p, p, None, 1, p, None) == -2         # ... per weight group
    assert L.w4a4_quantize_act(p, 4, 256, 256, 1, 128, p, p, p, None, 1, None, None) == -1     # ... and the token sums
    assert L.w4a4_quantize_act(p, 4, 64, 64, 0, 32, p, p, None, None, 1, p, None) == -2        # ... and no K-groups
    assert L.w4a4_quantize_act(p, 4, 64, 64, 0, 0, p, p, None, None, 5, p, None) == -1
    assert L.w4a4_quantize_weight(p, 4, 64, 0, 48, p, p, None, None, None, 0, None, None) == -2
    assert L.w4a4_quantize_weight(p, 4, 64, 0, 0, p, p, None, None, p, 0, None, None) == -1    # rowsum needs gsum
    assert L.w4a4_quantize_weight(p, 0, 64, 0, 0, p, p, None, None, None, 0, None, None) == 0
    assert L.w4a4_quantize_weight(p, 4, 64, 0, 0, p, p, None, None, None, 1, None, None) == -1 # operand layout needs esum
    assert L.w4a4_quantize_weight(p, 4, 64, 0, 32, p, p, None, None, None, 1, p, None) == -2


def test_linear_f16act_argument_errors(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)
    ep = b._Epilogue(None, 0, 0, 0, 0, 0, 0)

    def f(M=4, K=64, ldx=None, w=None, e=ep, x=p, o=p):
        w = _wt(b, K=K) if w is None else w
        return L.w4a4_linear_f16act(x, M, K, K if ldx is None else ldx, ctypes.byref(w), ctypes.byref(e), o, None)

    assert f(w=_wt(b, K=128)) == -1                                   # K mismatch
    assert f(ldx=32) == -1                                            # ldx < K
    assert f(x=None) == -1 and f(o=None) == -1                        # null pointers
    assert f(e=b._Epilogue(None, 7, 0, 0, 0, 0, 0)) == -1             # unknown activation
    assert f(K=96, w=_wt(b, K=96)) == -2                              # K % 64
    assert f(K=8192, w=_wt(b, K=8192)) == -2                          # K > 4096
    assert f(w=_wt(b, N=12)) == -2                                    # N % 8
    assert f(ldx=68) == -2                                            # rows not 16-byte aligned
    assert f(x=ctypes.c_void_p(0x1004)) == -2                         # misaligned
    assert f(w=_wt(b, mode=1)) == -2                                  # asymmetric weights
    assert f(K=256, w=_wt(b, K=256, group=128)) == -2                 # K-grouped weights
    assert f(K=256, w=_wt(b, K=256, layout=1, esum=0x3000)) == -2     # operand-layout weights
    assert f(e=b._Epilogue(None, 0, 1, 0, 0, 0, 0)) == -2             # requant is the two-call path's
    assert f(M=0) == 0


def test_layernorm_quantize_argument_errors(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)

    def f(M=4, K=64, ldx=None, x=p, r=None, g=p, be=p, eps=1e-5, y=None, mode=0, group=0, q=p, s=p, z=None,
          gs=None, layout=0, osum=None):
        return L.w4a4_layernorm_quantize(x, r, M, K, K if ldx is None else ldx, g, be, eps, y, mode, group, q, s, z,
                                         gs, layout, osum, None)

    assert f(x=None) == -1 and f(g=None) == -1 and f(be=None) == -1 and f(q=None) == -1 and f(s=None) == -1
    assert f(ldx=32) == -1                                            # ldx < K
    assert f(eps=-1.0) == -1 and f(eps=float("nan")) == -1
    assert f(mode=1) == -1                                            # asymmetric needs zero
    assert f(mode=3) == -1 and f(layout=4) == -1
    assert f(layout=1) == -1                                          # operand layout needs osum
    assert f(layout=1, mode=1, z=p, osum=p) == -1                     # ... and symmetric codes
    assert f(K=48) == -2                                              # K % 32
    assert f(K=8192) == -2                                            # K > 4096
    assert f(ldx=68) == -2                                            # rows not 16-byte aligned
    assert f(group=24) == -2                                          # group % 32
    assert f(K=96, group=64) == -2                                    # group must divide K
    assert f(K=192, group=96, mode=1, z=p, gs=p) == -2                # group sums need power-of-two chunk counts
    assert f(K=128, group=64, layout=1, osum=p) == -2                 # no K-groups in the operand layout
    assert f(x=ctypes.c_void_p(0x1004)) == -2                         # misaligned
    assert f(M=0) == 0


def test_int8_sibling_argument_errors(b):
    L = b.lib()
    p = ctypes.c_void_p(0x1000)
    ep = b._Epilogue(None, 0, 0, 0, 0, 0, 0)

    def lin(M=4, N=8, K=128, lda=None, a=p, sa=p, w=p, sw=p, e=ep, o=p):
        return L.w8a8_linear(a, K if lda is None else lda, sa, M, w, sw, N, K, ctypes.byref(e), o, None)

    assert lin(a=None) == -1 and lin(sa=None) == -1 and lin(w=None) == -1 and lin(sw=None) == -1 and lin(o=None) == -1
    assert lin(lda=64) == -1                                          # lda < K
    assert lin(e=b._Epilogue(None, 9, 0, 0, 0, 0, 0)) == -1           # unknown activation
    assert lin(e=b._Epilogue(None, 0, 1, 0, 0, 0, 0)) == -2           # no requantize here
    assert lin(K=96) == -2 and lin(K=64) == -2                        # K % 64, K >= 128
    assert lin(N=12) == -2 and lin(lda=136) == -2                     # N % 8, lda % 16
    assert lin(a=ctypes.c_void_p(0x1004)) == -2                       # misaligned
    assert lin(M=0) == 0
    assert L.w8a8_gemm_i32(p, 128, p, 4, p, p, 8, 128, None, None) == -1
    assert L.w8a8_quantize_rows(None, 4, 64, 64, p, p, None) == -1
    assert L.w8a8_quantize_rows(p, 4, 64, 32, p, p, None) == -1       # ldx < K
    assert L.w8a8_quantize_rows(p, 4, 48, 48, p, p, None) == -2       # K % 32
    assert L.w8a8_quantize_rows(p, 4, 32768, 32768, p, p, None) == -2
    assert L.w8a8_quantize_rows(p, 0, 64, 64, p, p, None) == 0
    ep0 = b._Epilogue(None, 0, 0, 0, 0, 0, 0)

    def f8(M=4, K=64, ldx=None, N=8, e=ep0, x=p, w=p, s_=p, o=p):
        return L.w8a8_linear_f16act(x, M, K, K if ldx is None else ldx, w, s_, N, ctypes.byref(e), o, None)

    assert f8(ldx=32) == -1 and f8(x=None) == -1 and f8(w=None) == -1 and f8(s_=None) == -1 and f8(o=None) == -1
    assert f8(e=b._Epilogue(None, 9, 0, 0, 0, 0, 0)) == -1
    assert f8(e=b._Epilogue(None, 0, 1, 0, 0, 0, 0)) == -2              # requant belongs to the INT4 path
    assert f8(K=96) == -2 and f8(K=8192) == -2 and f8(N=12) == -2 and f8(ldx=68) == -2
    assert f8(x=ctypes.c_void_p(0x1004)) == -2
    assert f8(M=0) == 0


def test_workspace_bytes(b):
    assert b.workspace_bytes(128, 768, 768, requant=False) == 0
    assert b.workspace_bytes(128, 768, 768, requant=True) == 128 * 768 * 4
