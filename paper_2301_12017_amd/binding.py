"""ctypes binding of libw4a4.so: argument marshalling only.

Every step of the W4A4 linear layer runs in the HIP kernels behind the C ABI
declared in include/w4a4.h; PyTorch appears here only as the owner of device
memory and of the stream the kernels are enqueued on.  There is no CPU or
PyTorch fallback: if the shared object is missing, loading fails.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

SYM, ASYM = 0, 1
ACT_NONE, ACT_GELU = 0, 1
LAYOUT_CANONICAL, LAYOUT_MFMA, LAYOUT_FP6 = 0, 1, 2


def _row_bytes(K, layout):
    """Bytes of a row of K codes: two per byte, or 3/4 byte each in the FP6 operand layout."""
    return K // 4 * 3 if layout == LAYOUT_FP6 else K // 2


def _rows_alloc(rows, layout, weight):
    """Rows to allocate for a matrix of codes: the FP6 operand layout stores whole panels (64 tokens, 128 channels)."""
    if layout != LAYOUT_FP6:
        return rows
    return (rows + 127) // 128 * 128 if weight else (rows + 63) // 64 * 64

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libw4a4.so")


class W4A4Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _Act(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("zero", ctypes.c_void_p),
                ("gsum", ctypes.c_void_p), ("M", ctypes.c_int), ("K", ctypes.c_int),
                ("lda", ctypes.c_int), ("group", ctypes.c_int), ("mode", ctypes.c_int),
                ("layout", ctypes.c_int), ("osum", ctypes.c_void_p), ("ldo", ctypes.c_int)]


class _Weight(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("zero", ctypes.c_void_p),
                ("rowsum_deq", ctypes.c_void_p), ("N", ctypes.c_int), ("K", ctypes.c_int),
                ("group", ctypes.c_int), ("mode", ctypes.c_int), ("layout", ctypes.c_int),
                ("esum", ctypes.c_void_p)]


class _Epilogue(ctypes.Structure):
    _fields_ = [("bias_f16", ctypes.c_void_p), ("act", ctypes.c_int), ("requant", ctypes.c_int),
                ("requant_mode", ctypes.c_int), ("requant_group", ctypes.c_int),
                ("requant_layout", ctypes.c_int), ("schedule", ctypes.c_int)]


class _Part(ctypes.Structure):
    _fields_ = [("w4", _Weight), ("w8q", ctypes.c_void_p), ("w8s", ctypes.c_void_p),
                ("bias_f16", ctypes.c_void_p), ("act", ctypes.c_int)]


class _StrategyCosts(ctypes.Structure):
    _fields_ = [("part_us", (ctypes.c_float * 2) * 4), ("ffn_fused_us", ctypes.c_float)]


class _LayerWeights(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int), ("heads", ctypes.c_int), ("ffn", ctypes.c_int),
                ("qkv", _Part), ("attn_out", _Part), ("ffn1", _Part), ("ffn2", _Part),
                ("ln1_gamma_f16", ctypes.c_void_p), ("ln1_beta_f16", ctypes.c_void_p),
                ("ln2_gamma_f16", ctypes.c_void_p), ("ln2_beta_f16", ctypes.c_void_p), ("ln_eps", ctypes.c_float)]


_lib = None

_vp, _i, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
_SIGNATURES = {
    "w4a4_version": (ctypes.c_char_p, []),
    "w4a4_status_string": (ctypes.c_char_p, [_i]),
    "w4a4_schedule_count": (_i, []),
    "w4a4_schedule_name": (ctypes.c_char_p, [_i]),
    "w4a4_preferred_layout": (_i, [_i, _i, _i, _i, _i]),
    "w4a4_time_next_gemm": (_i, [_vp, _vp]),
    "w4a4_workspace_bytes": (_sz, [_i, _i, _i, ctypes.POINTER(_Epilogue)]),
    "w4a4_linear_workspace_bytes": (_sz, [ctypes.POINTER(_Act), ctypes.POINTER(_Weight), ctypes.POINTER(_Epilogue), _i]),
    "w4a4_quantize_weight": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _i, _vp, _vp]),
    "w4a4_quantize_act": (_i, [_vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _i, _vp, _vp]),
    "w4a4_linear": (_i, [ctypes.POINTER(_Act), ctypes.POINTER(_Weight), ctypes.POINTER(_Epilogue),
                         _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "w4a4_linear_static": (_i, [ctypes.POINTER(_Act), ctypes.POINTER(_Weight), ctypes.POINTER(_Epilogue),
                                _vp, _vp, _vp, _vp, _vp]),
    "w8a8_quantize_rows": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp]),
    "w8a8_linear": (_i, [_vp, _i, _vp, _i, _vp, _vp, _i, _i, ctypes.POINTER(_Epilogue), _vp, _vp]),
    "w8a8_linear_f16act": (_i, [_vp, _i, _i, _i, _vp, _vp, _i, ctypes.POINTER(_Epilogue), _vp, _vp]),
    "w8a8_gemm_i32": (_i, [_vp, _i, _vp, _i, _vp, _vp, _i, _i, _vp, _vp]),
    "w4a4_layernorm_quantize": (_i, [_vp, _vp, _i, _i, _i, _vp, _vp, ctypes.c_float, _vp, _i, _i, _vp, _vp, _vp, _vp,
                                     _i, _vp, _vp]),
    "w4a4_linear_f16act": (_i, [_vp, _i, _i, _i, ctypes.POINTER(_Weight), ctypes.POINTER(_Epilogue), _vp, _vp]),
    "w4a4_part_workspace_bytes": (_sz, [_i, ctypes.POINTER(_Part)]),
    "w4a4_part_linear": (_i, [_vp, _i, _i, ctypes.POINTER(_Part), _i, _vp, _vp, _sz, _vp]),
    "w4a4_ffn_workspace_bytes": (_sz, [_i, ctypes.POINTER(_Part), ctypes.POINTER(_Part)]),
    "w4a4_ffn": (_i, [_vp, _i, _i, ctypes.POINTER(_Part), ctypes.POINTER(_Part), _i, _vp, _vp, _sz, _vp]),
    "w4a4_strategy_pick": (_i, [ctypes.POINTER(_StrategyCosts)]),
    "w4a4_strategy_tune": (_i, [_i, _i, _i, _i, ctypes.POINTER(_StrategyCosts), _vp]),
    "w4a4_strategy_lookup": (_i, [_i, _i, _i]),
    "w4a4_attention_f16": (_i, [_vp, _i, _i, _i, _vp, _vp]),
    "w4a4_encoder_layer_workspace_bytes": (_sz, [_i, _i, ctypes.POINTER(_LayerWeights)]),
    "w4a4_encoder_layer": (_i, [_vp, _i, _i, ctypes.POINTER(_LayerWeights), _i, _vp, _vp, _sz, _vp]),
    "w4a4_fused_fault_check": (_i, [_vp]),
    "w4a4_debug_fused_wait": (_i, [_i, _i]),
    "w4a4_probe_mfma": (ctypes.c_long, [_vp, _i, _vp, _vp]),
    "w4a4_probe_mfma_fp6": (ctypes.c_long, [_vp, _i, _vp, _vp]),
    "w4a4_probe_stream": (_i, [_vp, _vp, _sz, _vp, _vp]),
    "w4a4_pick_schedule": (_i, [ctypes.POINTER(_Act), ctypes.POINTER(_Weight), ctypes.POINTER(_Epilogue)]),
    "w4a4_gemm_i32": (_i, [ctypes.POINTER(_Act), ctypes.POINTER(_Weight), _vp, _i, _vp]),
    "w4a4_dequant_epilogue": (_i, [_vp, ctypes.POINTER(_Act), ctypes.POINTER(_Weight),
                                   ctypes.POINTER(_Epilogue), _vp, _vp, _vp, _vp, _vp]),
}
EXPORTS = tuple(_SIGNATURES)


def lib():
    """Load libw4a4.so (built by paper_2301_12017_amd/build.py).  Fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2301_12017_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


_hip = None


def _hiprt():
    """The HIP runtime this process already has loaded (for events only)."""
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(_vp)]
        _hip.hipEventDestroy.argtypes = [_vp]
        _hip.hipEventSynchronize.argtypes = [_vp]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), _vp, _vp]
    return _hip


class KernelTimer:
    """A pair of HIP events that w4a4_time_next_gemm stamps with the start and the end of the
    GEMM kernel of the next linear() / gemm_i32() call of this thread."""

    def __init__(self):
        self.start, self.stop = _vp(), _vp()
        for e in (self.start, self.stop):
            if _hiprt().hipEventCreate(ctypes.byref(e)) != 0:
                raise RuntimeError("hipEventCreate failed")

    def arm(self):
        _check(lib().w4a4_time_next_gemm(self.start, self.stop), "w4a4_time_next_gemm")

    def elapsed_ms(self) -> float:
        """Kernel duration; call after the stream has been synchronized."""
        ms = ctypes.c_float()
        rc = _hiprt().hipEventElapsedTime(ctypes.byref(ms), self.start, self.stop)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def __del__(self):
        try:
            for e in (self.start, self.stop):
                if e:
                    _hiprt().hipEventDestroy(e)
        except Exception:
            pass


def version() -> str:
    return lib().w4a4_version().decode()


def status_string(status: int) -> str:
    return lib().w4a4_status_string(int(status)).decode()


def schedule_names():
    L = lib()
    return [L.w4a4_schedule_name(i + 1).decode() for i in range(L.w4a4_schedule_count())]


def schedule_number(name: str) -> int:
    """1-based number of the schedule called `name` (what w4a4_epilogue.schedule takes)."""
    return schedule_names().index(name) + 1


def fused_fault_check() -> bool:
    """w4a4_fused_fault_check on the current stream: True if a fused requantize gave up since the last check."""
    rc = lib().w4a4_fused_fault_check(_stream())
    if rc < 0:
        raise W4A4Error(rc, "w4a4_fused_fault_check")
    return bool(rc)


def debug_fused_wait(spin_limit: int = 0, extra_arrivals: int = 0):
    _check(lib().w4a4_debug_fused_wait(spin_limit, extra_arrivals), "w4a4_debug_fused_wait")


def pick_schedule(A: "QAct", W: "QWeight", requant=False, requant_mode=SYM, requant_group=0, schedule=0,
                  requant_layout=LAYOUT_CANONICAL) -> str:
    """Name of the schedule w4a4_linear runs this layer on."""
    ep = _Epilogue(None, 0, int(requant), requant_mode, requant_group, requant_layout, schedule)
    a, w = A.c(), W.c()
    rc = lib().w4a4_pick_schedule(ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep))
    if rc < 0:
        raise W4A4Error(rc, "w4a4_pick_schedule")
    return schedule_names()[rc - 1]


def probe_mfma(operands: torch.Tensor, iters: int, sink: torch.Tensor) -> int:
    """w4a4_probe_mfma; returns the number of wave-level MFMA instructions the launch issues."""
    assert operands.dtype == torch.int32 and operands.numel() == 64 * 16 and operands.is_cuda
    n = lib().w4a4_probe_mfma(_ptr(operands), iters, _ptr(sink), _stream())
    if n < 0:
        raise W4A4Error(int(n), "w4a4_probe_mfma")
    return int(n)


def probe_mfma_fp6(operands: torch.Tensor, iters: int, sink: torch.Tensor) -> int:
    """w4a4_probe_mfma_fp6; returns the number of wave-level MFMA instructions the launch issues."""
    assert operands.dtype == torch.int32 and operands.numel() == 64 * 32 and operands.is_cuda
    n = lib().w4a4_probe_mfma_fp6(_ptr(operands), iters, _ptr(sink), _stream())
    if n < 0:
        raise W4A4Error(int(n), "w4a4_probe_mfma_fp6")
    return int(n)


def probe_stream(src: torch.Tensor, dst: Optional[torch.Tensor], sink: torch.Tensor):
    _check(lib().w4a4_probe_stream(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _ptr(sink), _stream()),
           "w4a4_probe_stream")


def preferred_layout(M: int, N: int, K: int, mode=SYM, group=0) -> int:
    return int(lib().w4a4_preferred_layout(M, N, K, mode, group))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise W4A4Error(rc, where)


@dataclass
class QAct:
    """Token-wise quantized activations on the device (see w4a4_act in include/w4a4.h)."""
    q: torch.Tensor
    scale: torch.Tensor
    zero: Optional[torch.Tensor]
    gsum: Optional[torch.Tensor]
    M: int
    K: int
    lda: int
    group: int
    mode: int
    q_offset_bytes: int = 0     # column-slice view: start this many bytes into each row
    layout: int = LAYOUT_CANONICAL
    osum: Optional[torch.Tensor] = None   # [M, slices] odd-position code sums (MFMA operand layout)
    osum_index: int = 0         # which slice of osum this view covers

    def c(self) -> _Act:
        osum, ldo = None, 1
        if self.osum is not None:
            ldo = 1 if (self.osum.dim() == 1 or self.mode == ASYM) else self.osum.shape[1]
            osum = self.osum.data_ptr() + 4 * self.osum_index
        return _Act(self.q.data_ptr() + self.q_offset_bytes, self.scale.data_ptr(),
                    None if self.zero is None else self.zero.data_ptr(),
                    None if self.gsum is None else self.gsum.data_ptr(),
                    self.M, self.K, self.lda, self.group, self.mode, self.layout, osum, ldo)


@dataclass
class QWeight:
    """Offline-quantized weights on the device (see w4a4_weight in include/w4a4.h)."""
    q: torch.Tensor
    scale: torch.Tensor
    zero: Optional[torch.Tensor]
    gsum: Optional[torch.Tensor]
    rowsum_deq: Optional[torch.Tensor]
    N: int
    K: int
    group: int
    mode: int
    layout: int = LAYOUT_CANONICAL
    esum: Optional[torch.Tensor] = None   # [N] even-position code sums (MFMA operand layout)

    def c(self) -> _Weight:
        return _Weight(self.q.data_ptr(), self.scale.data_ptr(),
                       None if self.zero is None else self.zero.data_ptr(),
                       None if self.rowsum_deq is None else self.rowsum_deq.data_ptr(),
                       self.N, self.K, self.group, self.mode, self.layout,
                       None if self.esum is None else self.esum.data_ptr())


def _ng(K, group):
    return 1 if group == 0 else K // group


def quantize_weight(W: torch.Tensor, mode=SYM, group=0, layout=LAYOUT_CANONICAL) -> QWeight:
    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous()
    N, K = W.shape
    ng = _ng(K, group)
    dev = W.device
    q = torch.empty((_rows_alloc(N, layout, True), _row_bytes(K, layout)), dtype=torch.uint8, device=dev)
    scale = torch.empty((N, ng), dtype=torch.float32, device=dev)
    zero = torch.empty((N, ng), dtype=torch.float32, device=dev) if mode == ASYM else None
    gsum = torch.empty((N, ng), dtype=torch.int32, device=dev)
    c = torch.empty((N,), dtype=torch.float32, device=dev)
    esum = None
    if layout == LAYOUT_MFMA:                             # layout-private sums: [N] (symmetric) or [N, ng + 1] (unsigned)
        esum = torch.empty((N,) if mode == SYM else (N, ng + 1), dtype=torch.int32, device=dev)
    rc = lib().w4a4_quantize_weight(_ptr(W), N, K, mode, group, _ptr(q), _ptr(scale), _ptr(zero),
                                    _ptr(gsum), _ptr(c), layout, _ptr(esum), _stream())
    _check(rc, "w4a4_quantize_weight")
    return QWeight(q, scale, zero, gsum, c, N, K, group, mode, layout, esum)


def quantize_act(X: torch.Tensor, mode=SYM, group=0, out: Optional[QAct] = None,
                 layout=LAYOUT_CANONICAL) -> QAct:
    assert X.is_cuda and X.dtype == torch.float16 and X.stride(1) == 1
    M, K = X.shape
    ng = _ng(K, group)
    dev = X.device
    if out is None:
        out = QAct(torch.empty((_rows_alloc(M, layout, False), _row_bytes(K, layout)), dtype=torch.uint8, device=dev),
                   torch.empty((M,), dtype=torch.float32, device=dev),
                   torch.empty((M,), dtype=torch.float32, device=dev) if mode == ASYM else None,
                   torch.empty((M, ng), dtype=torch.int32, device=dev) if mode == ASYM else None,
                   M, K, _row_bytes(K, layout), group, mode, 0, layout, _new_osum(M, ng, mode, layout, dev))
    rc = lib().w4a4_quantize_act(_ptr(X), M, K, X.stride(0), mode, group, _ptr(out.q), _ptr(out.scale),
                                 _ptr(out.zero), _ptr(out.gsum), out.layout, _ptr(out.osum), _stream())
    _check(rc, "w4a4_quantize_act")
    return out


def _new_qact(M, K, mode, group, layout, dev) -> QAct:
    ng = _ng(K, group)
    return QAct(torch.empty((_rows_alloc(M, layout, False), _row_bytes(K, layout)), dtype=torch.uint8, device=dev),
                torch.empty((M,), dtype=torch.float32, device=dev),
                torch.empty((M,), dtype=torch.float32, device=dev) if mode == ASYM else None,
                torch.empty((M, ng), dtype=torch.int32, device=dev) if mode == ASYM else None,
                M, K, _row_bytes(K, layout), group, mode, 0, layout, _new_osum(M, ng, mode, layout, dev))


def _new_osum(M, ng, mode, layout, dev):
    """Layout-private token sums of the MFMA operand layout: [M] odd-position sums (symmetric codes), or [ng, M]
    = 128 x the even-position sums of every weight group (unsigned codes)."""
    if layout != LAYOUT_MFMA:
        return None
    return torch.empty((M,) if mode == SYM else (ng, M), dtype=torch.int32, device=dev)


def layernorm_quantize(X: torch.Tensor, R: Optional[torch.Tensor], gamma: torch.Tensor, beta: torch.Tensor,
                       eps: float, mode=SYM, group=0, layout=LAYOUT_CANONICAL, want_y=True,
                       out: Optional[QAct] = None, y: Optional[torch.Tensor] = None):
    """w4a4_layernorm_quantize: (QAct of LayerNorm(X + R) * gamma + beta, its fp16 copy or None)."""
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    assert R is None or (R.dtype == torch.float16 and R.shape == X.shape and R.stride() == X.stride())
    M, K = X.shape
    if out is None:
        out = _new_qact(M, K, mode, group, layout, X.device)
    if y is None and want_y:
        y = torch.empty((M, K), dtype=torch.float16, device=X.device)
    rc = lib().w4a4_layernorm_quantize(_ptr(X), _ptr(R), M, K, X.stride(0), _ptr(gamma), _ptr(beta), float(eps),
                                       _ptr(y), mode, group, _ptr(out.q), _ptr(out.scale), _ptr(out.zero),
                                       _ptr(out.gsum), out.layout, _ptr(out.osum), _stream())
    _check(rc, "w4a4_layernorm_quantize")
    return out, y


class PreparedLayerNormQuantize:
    """A w4a4_layernorm_quantize call with its arguments marshalled once (see PreparedLinear)."""

    def __init__(self, X, R, gamma, beta, eps, out: QAct, y=None):
        M, K = X.shape
        self.keep = (X, R, gamma, beta, out, y)
        self.args = (_ptr(X), _ptr(R), M, K, X.stride(0), _ptr(gamma), _ptr(beta), float(eps), _ptr(y), out.mode,
                     out.group, _ptr(out.q), _ptr(out.scale), _ptr(out.zero), _ptr(out.gsum), out.layout,
                     _ptr(out.osum))
        self.fn = lib().w4a4_layernorm_quantize

    def __call__(self, stream=None):
        rc = self.fn(*self.args, _stream() if stream is None else stream)
        if rc:
            raise W4A4Error(rc, "w4a4_layernorm_quantize")


def workspace_bytes(M, N, K, requant=False) -> int:
    ep = _Epilogue(None, 0, int(requant), 0, 0, 0, 0)
    return int(lib().w4a4_workspace_bytes(M, N, K, ctypes.byref(ep)))


def linear_workspace_bytes(A: "QAct", W: "QWeight", requant=True, requant_mode=SYM, requant_group=0,
                           want_gsum=False, schedule=0, requant_layout=LAYOUT_CANONICAL) -> int:
    ep = _Epilogue(None, 0, int(requant), requant_mode, requant_group, requant_layout, schedule)
    want_gsum = want_gsum or requant_layout == LAYOUT_MFMA
    a, w = A.c(), W.c()
    return int(lib().w4a4_linear_workspace_bytes(ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep), int(want_gsum)))


def fused_fault(workspace: torch.Tensor, nbytes: int) -> int:
    """Last word of a fused requantize workspace of `nbytes` bytes, the size w4a4_linear_workspace_bytes gave
    for the layer (0 = the row-maximum exchange completed)."""
    return int(workspace[:nbytes].view(torch.int32)[-1].item())


def _epilogue(bias, act, requant, requant_mode, requant_group, schedule, requant_layout=LAYOUT_CANONICAL):
    return _Epilogue(None if bias is None else bias.data_ptr(), act, int(bool(requant)), requant_mode,
                     requant_group, requant_layout, schedule)


def _alloc_out(A: QAct, W: QWeight, requant, requant_mode, requant_group, requant_layout=LAYOUT_CANONICAL):
    dev = A.q.device
    if not requant:
        return torch.empty((A.M, W.N), dtype=torch.float16, device=dev), None, None, None
    rng = _ng(W.N, requant_group)
    sums = requant_mode == ASYM or requant_layout == LAYOUT_MFMA
    return (torch.empty((_rows_alloc(A.M, requant_layout, False), _row_bytes(W.N, requant_layout)), dtype=torch.uint8, device=dev),
            torch.empty((A.M,), dtype=torch.float32, device=dev),
            torch.empty((A.M,), dtype=torch.float32, device=dev) if requant_mode == ASYM else None,
            torch.empty((A.M, rng), dtype=torch.int32, device=dev) if sums else None)


def linear(A: QAct, W: QWeight, bias: Optional[torch.Tensor] = None, act=ACT_NONE, requant=False,
           requant_mode=SYM, requant_group=0, schedule=0, out=None, workspace: Optional[torch.Tensor] = None,
           requant_layout=LAYOUT_CANONICAL):
    """w4a4_linear.  Returns an fp16 tensor [M,N], or a QAct holding the requantized output."""
    ep = _epilogue(bias, act, requant, requant_mode, requant_group, schedule, requant_layout)
    if out is None:
        out = _alloc_out(A, W, requant, requant_mode, requant_group, requant_layout)
    o, os_, oz, og = out
    a, w = A.c(), W.c()
    need = int(lib().w4a4_linear_workspace_bytes(ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep),
                                                 0 if og is None else 1))
    if need and workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=A.q.device)
    rc = lib().w4a4_linear(ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep), _ptr(o), _ptr(os_), _ptr(oz),
                           _ptr(og), _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream())
    _check(rc, "w4a4_linear")
    if not requant:
        return o
    if requant_layout == LAYOUT_MFMA:
        return QAct(o, os_, oz, None, A.M, W.N, W.N // 2, requant_group, requant_mode, 0, LAYOUT_MFMA, og)
    if requant_layout == LAYOUT_FP6:
        return QAct(o, os_, None, None, A.M, W.N, _row_bytes(W.N, LAYOUT_FP6), requant_group, requant_mode, 0, LAYOUT_FP6, None)
    return QAct(o, os_, oz, og, A.M, W.N, W.N // 2, requant_group, requant_mode)


def linear_static(A: QAct, W: QWeight, bias: Optional[torch.Tensor] = None, act=ACT_NONE, requant=False,
                  requant_mode=SYM, requant_group=0, schedule=0, out=None, requant_layout=LAYOUT_CANONICAL):
    """w4a4_linear_static: w4a4_linear without a workspace argument (the library's static exchange area).
    `out` as for linear(); when it is given this wrapper allocates nothing either."""
    ep = _epilogue(bias, act, requant, requant_mode, requant_group, schedule, requant_layout)
    if out is None:
        out = _alloc_out(A, W, requant, requant_mode, requant_group, requant_layout)
    o, os_, oz, og = out
    a, w = A.c(), W.c()
    rc = lib().w4a4_linear_static(ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep), _ptr(o), _ptr(os_), _ptr(oz),
                                  _ptr(og), _stream())
    _check(rc, "w4a4_linear_static")
    if not requant:
        return o
    if requant_layout == LAYOUT_MFMA:
        return QAct(o, os_, oz, None, A.M, W.N, W.N // 2, requant_group, requant_mode, 0, LAYOUT_MFMA, og)
    if requant_layout == LAYOUT_FP6:
        return QAct(o, os_, None, None, A.M, W.N, _row_bytes(W.N, LAYOUT_FP6), requant_group, requant_mode, 0, LAYOUT_FP6, None)
    return QAct(o, os_, oz, og, A.M, W.N, W.N // 2, requant_group, requant_mode)


class PreparedLinear:
    """A w4a4_linear call with every argument marshalled once: calling the object only makes the
    C call on the current stream.  For loops that must not be slowed down by Python (benchmarks,
    graph capture).  The tensors it was built from are kept alive."""

    def __init__(self, A: QAct, W: QWeight, bias=None, act=ACT_NONE, requant=False, requant_mode=SYM,
                 requant_group=0, schedule=0, out=None, workspace=None, requant_layout=LAYOUT_CANONICAL):
        self.keep = (A, W, bias, out, workspace)
        self.ep = _epilogue(bias, act, requant, requant_mode, requant_group, schedule, requant_layout)
        if out is None:
            out = _alloc_out(A, W, requant, requant_mode, requant_group, requant_layout)
        self.out = out
        self.a, self.w = A.c(), W.c()
        need = int(lib().w4a4_linear_workspace_bytes(ctypes.byref(self.a), ctypes.byref(self.w),
                                                     ctypes.byref(self.ep), 0 if out[3] is None else 1))
        if need and workspace is None:
            workspace = torch.empty((need,), dtype=torch.uint8, device=A.q.device)
        self.workspace = workspace
        self.args = (ctypes.byref(self.a), ctypes.byref(self.w), ctypes.byref(self.ep), _ptr(out[0]), _ptr(out[1]),
                     _ptr(out[2]), _ptr(out[3]), _ptr(workspace), 0 if workspace is None else workspace.numel())
        self.fn = lib().w4a4_linear

    def __call__(self, stream=None):
        rc = self.fn(*self.args, _stream() if stream is None else stream)
        if rc:
            raise W4A4Error(rc, "w4a4_linear")


def linear_f16act(X: torch.Tensor, W: QWeight, bias: Optional[torch.Tensor] = None, act=ACT_NONE,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """w4a4_linear_f16act: quantize_act + linear in one kernel, for small token counts.  fp16 [M,N]."""
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    if out is None:
        out = torch.empty((M, W.N), dtype=torch.float16, device=X.device)
    ep, w = _epilogue(bias, act, False, SYM, 0, 0, LAYOUT_CANONICAL), W.c()
    rc = lib().w4a4_linear_f16act(_ptr(X), M, K, X.stride(0), ctypes.byref(w), ctypes.byref(ep), _ptr(out), _stream())
    _check(rc, "w4a4_linear_f16act")
    return out


# ---- the INT8 sibling -------------------------------------------------------------------------------
def quantize_rows8(X: torch.Tensor, q: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None):
    """w8a8_quantize_rows: (int8 codes [M,K], fp32 scales [M]) of fp16 rows (tokens, or weight channels)."""
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    q = torch.empty((M, K), dtype=torch.int8, device=X.device) if q is None else q
    scale = torch.empty((M,), dtype=torch.float32, device=X.device) if scale is None else scale
    _check(lib().w8a8_quantize_rows(_ptr(X), M, K, X.stride(0), _ptr(q), _ptr(scale), _stream()), "w8a8_quantize_rows")
    return q, scale


def linear8(Aq, sa, Wq, sw, bias=None, act=ACT_NONE, out=None):
    """w8a8_linear: fp16 [M,N]."""
    M, K = Aq.shape
    N = Wq.shape[0]
    out = torch.empty((M, N), dtype=torch.float16, device=Aq.device) if out is None else out
    ep = _epilogue(bias, act, False, SYM, 0, 0, LAYOUT_CANONICAL)
    rc = lib().w8a8_linear(_ptr(Aq), Aq.stride(0), _ptr(sa), M, _ptr(Wq), _ptr(sw), N, K, ctypes.byref(ep), _ptr(out),
                           _stream())
    _check(rc, "w8a8_linear")
    return out


def linear8_f16act(X, Wq, sw, bias=None, act=ACT_NONE, out=None):
    """w8a8_linear_f16act: fp16 [M,N] from fp16 activations in one kernel (small token counts)."""
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    M, K = X.shape
    N = Wq.shape[0]
    out = torch.empty((M, N), dtype=torch.float16, device=X.device) if out is None else out
    ep = _epilogue(bias, act, False, SYM, 0, 0, LAYOUT_CANONICAL)
    rc = lib().w8a8_linear_f16act(_ptr(X), M, K, X.stride(0), _ptr(Wq), _ptr(sw), N, ctypes.byref(ep), _ptr(out), _stream())
    _check(rc, "w8a8_linear_f16act")
    return out


def gemm8_i32(Aq, sa, Wq, sw):
    M, K = Aq.shape
    N = Wq.shape[0]
    acc = torch.empty((M, N), dtype=torch.int32, device=Aq.device)
    rc = lib().w8a8_gemm_i32(_ptr(Aq), Aq.stride(0), _ptr(sa), M, _ptr(Wq), _ptr(sw), N, K, _ptr(acc), _stream())
    _check(rc, "w8a8_gemm_i32")
    return acc


class PreparedLinear8:
    """A w8a8_linear call with its arguments marshalled once (see PreparedLinear)."""

    def __init__(self, Aq, sa, Wq, sw, bias=None, act=ACT_NONE, out=None):
        M, K = Aq.shape
        N = Wq.shape[0]
        self.out = torch.empty((M, N), dtype=torch.float16, device=Aq.device) if out is None else out
        self.keep = (Aq, sa, Wq, sw, bias)
        self.ep = _epilogue(bias, act, False, SYM, 0, 0, LAYOUT_CANONICAL)
        self.args = (_ptr(Aq), Aq.stride(0), _ptr(sa), M, _ptr(Wq), _ptr(sw), N, K, ctypes.byref(self.ep), _ptr(self.out))
        self.fn = lib().w8a8_linear

    def __call__(self, stream=None):
        rc = self.fn(*self.args, _stream() if stream is None else stream)
        if rc:
            raise W4A4Error(rc, "w8a8_linear")


class PreparedQuantizeRows8:
    def __init__(self, X, q, scale):
        M, K = X.shape
        self.keep = (X, q, scale)
        self.args = (_ptr(X), M, K, X.stride(0), _ptr(q), _ptr(scale))
        self.fn = lib().w8a8_quantize_rows

    def __call__(self, stream=None):
        rc = self.fn(*self.args, _stream() if stream is None else stream)
        if rc:
            raise W4A4Error(rc, "w8a8_quantize_rows")


# ---- per-part strategy -------------------------------------------------------------------------------
PART_QKV, PART_ATTN_OUT, PART_FFN1, PART_FFN2 = range(4)
STRATEGY_FUSED_FFN, STRATEGY_ALL_INT4 = 16, 31


class Part:
    """One linear part with its weights prepared in both precisions (w4a4_part in include/w4a4.h).
    The INT4 weights take the layout the library prefers for M tokens, or the one asked for."""

    def __init__(self, W: torch.Tensor, M: int, bias: Optional[torch.Tensor] = None, act=ACT_NONE, mode=SYM, group=0,
                 layout: Optional[int] = None):
        N, K = W.shape
        self.w4 = quantize_weight(W, mode, group, preferred_layout(M, N, K, mode, group) if layout is None else layout)
        self.w8q, self.w8s = quantize_rows8(W)
        self.bias, self.act, self.N, self.K = bias, act, N, K

    def c(self) -> _Part:
        return _Part(self.w4.c(), _ptr(self.w8q), _ptr(self.w8s), _ptr(self.bias), self.act)


def _workspace(nbytes: int, dev) -> torch.Tensor:
    return torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=dev)


def part_linear(X: torch.Tensor, P: Part, int4: bool, out=None, workspace=None) -> torch.Tensor:
    """w4a4_part_linear: fp16 [M, N] of part P in INT4 or in INT8."""
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    M = X.shape[0]
    c = P.c()
    need = lib().w4a4_part_workspace_bytes(M, ctypes.byref(c))
    workspace = _workspace(need, X.device) if workspace is None else workspace
    out = torch.empty((M, P.N), dtype=torch.float16, device=X.device) if out is None else out
    rc = lib().w4a4_part_linear(_ptr(X), M, X.stride(0), ctypes.byref(c), int(bool(int4)), _ptr(out), _ptr(workspace),
                                workspace.numel(), _stream())
    _check(rc, "w4a4_part_linear")
    return out


def ffn(X: torch.Tensor, P1: Part, P2: Part, strategy: int, out=None, workspace=None) -> torch.Tensor:
    """w4a4_ffn: FFN1 then FFN2 under `strategy` (bits PART_FFN1, PART_FFN2, STRATEGY_FUSED_FFN)."""
    assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
    M = X.shape[0]
    c1, c2 = P1.c(), P2.c()
    need = lib().w4a4_ffn_workspace_bytes(M, ctypes.byref(c1), ctypes.byref(c2))
    workspace = _workspace(need, X.device) if workspace is None else workspace
    out = torch.empty((M, P2.N), dtype=torch.float16, device=X.device) if out is None else out
    rc = lib().w4a4_ffn(_ptr(X), M, X.stride(0), ctypes.byref(c1), ctypes.byref(c2), strategy, _ptr(out),
                        _ptr(workspace), workspace.numel(), _stream())
    _check(rc, "w4a4_ffn")
    return out


def _costs_struct(part_us, ffn_fused_us) -> _StrategyCosts:
    c = _StrategyCosts()
    for p in range(4):
        for k in range(2):
            c.part_us[p][k] = part_us[p][k]
    c.ffn_fused_us = ffn_fused_us
    return c


def strategy_pick(part_us, ffn_fused_us) -> int:
    """w4a4_strategy_pick on a 4 x 2 table of microseconds ([part][0] INT8, [part][1] INT4)."""
    c = _costs_struct(part_us, ffn_fused_us)
    rc = lib().w4a4_strategy_pick(ctypes.byref(c))
    _check(min(rc, 0), "w4a4_strategy_pick")
    return rc


def strategy_tune(M: int, hidden: int, ffn_size: int, iters: int = 20):
    """w4a4_strategy_tune: (strategy, part_us [4][2], ffn_fused_us) measured on the current device."""
    c = _StrategyCosts()
    rc = lib().w4a4_strategy_tune(M, hidden, ffn_size, iters, ctypes.byref(c), _stream())
    _check(min(rc, 0), "w4a4_strategy_tune")
    return rc, [[c.part_us[p][k] for k in range(2)] for p in range(4)], c.ffn_fused_us


def strategy_lookup(M: int, hidden: int, ffn_size: int) -> int:
    rc = lib().w4a4_strategy_lookup(M, hidden, ffn_size)
    _check(min(rc, 0), "w4a4_strategy_lookup")
    return rc


# ---- whole encoder layer -----------------------------------------------------------------------------
STRATEGY_FUSED_LN = 32


def attention(QKV: torch.Tensor, batch: int, seq: int, heads: int, out=None) -> torch.Tensor:
    """w4a4_attention_f16: fp16 [batch*seq, heads*64] from fp16 [batch*seq, 3*heads*64]."""
    assert QKV.is_cuda and QKV.dtype == torch.float16 and QKV.is_contiguous() and QKV.shape == (batch * seq, 3 * heads * 64)
    out = torch.empty((batch * seq, heads * 64), dtype=torch.float16, device=QKV.device) if out is None else out
    _check(lib().w4a4_attention_f16(_ptr(QKV), batch, seq, heads, _ptr(out), _stream()), "w4a4_attention_f16")
    return out


class EncoderLayer:
    """The weights of one encoder layer (w4a4_encoder_layer_weights) and a workspace for `batch` x `seq` tokens."""

    def __init__(self, batch, seq, heads, Wqkv, bqkv, Wao, bao, W1, b1, W2, b2, g1, be1, g2, be2, eps=1e-12,
                 layout: Optional[int] = None):
        M = batch * seq
        self.batch, self.seq, self.heads, self.hidden, self.ffn = batch, seq, heads, Wao.shape[0], W1.shape[0]
        self.qkv, self.attn_out = Part(Wqkv, M, bqkv, layout=layout), Part(Wao, M, bao, layout=layout)
        self.ffn1, self.ffn2 = Part(W1, M, b1, ACT_GELU, layout=layout), Part(W2, M, b2, layout=layout)
        self.ln = (g1, be1, g2, be2)
        self.c = _LayerWeights(self.hidden, heads, self.ffn, self.qkv.c(), self.attn_out.c(), self.ffn1.c(), self.ffn2.c(),
                               _ptr(g1), _ptr(be1), _ptr(g2), _ptr(be2), eps)
        need = lib().w4a4_encoder_layer_workspace_bytes(batch, seq, ctypes.byref(self.c))
        if need == 0:
            raise W4A4Error(-1, "w4a4_encoder_layer_workspace_bytes")
        self.workspace = _workspace(need, Wqkv.device)

    def __call__(self, X: torch.Tensor, strategy: int, out=None, stream=None) -> torch.Tensor:
        assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.shape == (self.batch * self.seq, self.hidden)
        out = torch.empty_like(X) if out is None else out
        rc = lib().w4a4_encoder_layer(_ptr(X), self.batch, self.seq, ctypes.byref(self.c), strategy, _ptr(out),
                                      _ptr(self.workspace), self.workspace.numel(), _stream() if stream is None else stream)
        _check(rc, "w4a4_encoder_layer")
        return out


class PreparedLinearF16Act:
    """A w4a4_linear_f16act call with its arguments marshalled once (see PreparedLinear)."""

    def __init__(self, X: torch.Tensor, W: QWeight, bias=None, act=ACT_NONE, out=None):
        assert X.is_cuda and X.dtype == torch.float16 and X.dim() == 2 and X.stride(1) == 1
        M, K = X.shape
        if out is None:
            out = torch.empty((M, W.N), dtype=torch.float16, device=X.device)
        self.out = out
        self.keep = (X, W, bias, out)
        self.ep, self.w = _epilogue(bias, act, False, SYM, 0, 0, LAYOUT_CANONICAL), W.c()
        self.args = (_ptr(X), M, K, X.stride(0), ctypes.byref(self.w), ctypes.byref(self.ep), _ptr(out))
        self.fn = lib().w4a4_linear_f16act

    def __call__(self, stream=None):
        rc = self.fn(*self.args, _stream() if stream is None else stream)
        if rc:
            raise W4A4Error(rc, "w4a4_linear_f16act")


class PreparedQuantizeAct:
    """A w4a4_quantize_act call with its arguments marshalled once (see PreparedLinear)."""

    def __init__(self, X: torch.Tensor, out: QAct):
        assert X.is_cuda and X.dtype == torch.float16 and X.stride(1) == 1
        self.keep = (X, out)
        M, K = X.shape
        self.args = (_ptr(X), M, K, X.stride(0), out.mode, out.group, _ptr(out.q), _ptr(out.scale), _ptr(out.zero),
                     _ptr(out.gsum), out.layout, _ptr(out.osum))
        self.fn = lib().w4a4_quantize_act

    def __call__(self, stream=None):
        rc = self.fn(*self.args, _stream() if stream is None else stream)
        if rc:
            raise W4A4Error(rc, "w4a4_quantize_act")


def gemm_i32(A: QAct, W: QWeight, schedule=0) -> torch.Tensor:
    """w4a4_gemm_i32: int32 accumulators [ng, M, N]."""
    ng = _ng(W.K, W.group)
    acc = torch.empty((ng, A.M, W.N), dtype=torch.int32, device=A.q.device)
    a, w = A.c(), W.c()
    rc = lib().w4a4_gemm_i32(ctypes.byref(a), ctypes.byref(w), _ptr(acc), schedule, _stream())
    _check(rc, "w4a4_gemm_i32")
    return acc


def dequant_epilogue(acc: torch.Tensor, A: QAct, W: QWeight, bias=None, act=ACT_NONE, requant=False,
                     requant_mode=SYM, requant_group=0):
    """w4a4_dequant_epilogue on accumulators from gemm_i32."""
    ep = _epilogue(bias, act, requant, requant_mode, requant_group, 0)
    o, os_, oz, og = _alloc_out(A, W, requant, requant_mode, requant_group)
    a, w = A.c(), W.c()
    rc = lib().w4a4_dequant_epilogue(_ptr(acc), ctypes.byref(a), ctypes.byref(w), ctypes.byref(ep), _ptr(o),
                                     _ptr(os_), _ptr(oz), _ptr(og), _stream())
    _check(rc, "w4a4_dequant_epilogue")
    if not requant:
        return o
    return QAct(o, os_, oz, og, A.M, W.N, W.N // 2, requant_group, requant_mode)
