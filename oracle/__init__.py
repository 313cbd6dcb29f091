"""NumPy face of the CPU oracle (oracle/w4a4_oracle.c) plus an fp64 yardstick.

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this package; the GPU library and its
Python binding never do, and this package imports nothing of theirs.

Each wrapper allocates the output arrays, calls one C function and returns
them; no arithmetic of the method happens in Python here, except `truth64`,
which is a second, independent evaluation of the layer in float64 from the
dequantized operands (Sec. 3.1: x_q = S*code (+ x_zero)) used to pin the fp32
dequantize algebra and as the yardstick of the 1e-2 accuracy criterion.
"""
import ctypes
import math
import os

import numpy as np

from . import build as _build

SYM, ASYM = 0, 1
ACT_NONE, ACT_GELU = 0, 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = ctypes.CDLL(path)
        L.orc_h2f.restype = ctypes.c_float
        L.orc_h2f.argtypes = [ctypes.c_uint16]
        L.orc_f2h.restype = ctypes.c_uint16
        L.orc_f2h.argtypes = [ctypes.c_float]
        L.orc_gelu.restype = ctypes.c_float
        L.orc_gelu.argtypes = [ctypes.c_float]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ng(K, group):
    G = K if group == 0 else group
    if G <= 0 or K % G:
        raise ValueError("group must divide K")
    return K // G


# ------------------------------------------------------------------ scalars
def h2f(bits: int) -> float:
    return float(lib().orc_h2f(int(bits) & 0xFFFF))


def f2h(x: float) -> int:
    return int(lib().orc_f2h(ctypes.c_float(x)))


def gelu(x: float) -> float:
    return float(lib().orc_gelu(ctypes.c_float(x)))


# ------------------------------------------------------------------ vectors
def quant_sym(v):
    v = _c(v, np.float32)
    q = np.empty(v.size, np.int8)
    S = ctypes.c_float()
    lib().orc_quant_sym(_p(v), ctypes.c_int(v.size), _p(q), ctypes.byref(S))
    return q, np.float32(S.value)


def quant_asym(v):
    v = _c(v, np.float32)
    q = np.empty(v.size, np.uint8)
    S, Z = ctypes.c_float(), ctypes.c_float()
    lib().orc_quant_asym(_p(v), ctypes.c_int(v.size), _p(q), ctypes.byref(S), ctypes.byref(Z))
    return q, np.float32(S.value), np.float32(Z.value)


def pack(codes):
    codes = np.ascontiguousarray(codes).astype(np.int8)
    assert codes.size % 2 == 0
    out = np.empty(codes.size // 2, np.uint8)
    lib().orc_pack(_p(codes), ctypes.c_int(codes.size), _p(out))
    return out


def unpack(packed, mode):
    packed = _c(packed, np.uint8)
    flat = packed.reshape(-1)
    n = flat.size * 2
    if mode == SYM:
        out = np.empty(n, np.int8)
        lib().orc_unpack_signed(_p(flat), ctypes.c_int(n), _p(out))
    else:
        out = np.empty(n, np.uint8)
        lib().orc_unpack_unsigned(_p(flat), ctypes.c_int(n), _p(out))
    return out.reshape(packed.shape[:-1] + (packed.shape[-1] * 2,))


# ------------------------------------------------------------------ steps
def quantize_act(X_f16, mode=SYM, group=0):
    """X_f16: float16 [M, K] -> dict(q u8 [M,K/2], s f32 [M], z f32 [M], gsum i32 [M,ng])."""
    X = _c(X_f16, np.float16)
    M, K = X.shape
    ng = _ng(K, group)
    q = np.empty((M, K // 2), np.uint8)
    s = np.empty(M, np.float32)
    z = np.zeros(M, np.float32)
    gs = np.empty((M, ng), np.int32)
    rc = lib().orc_quantize_act(_p(X.view(np.uint16)), M, K, K, mode, group, _p(q), _p(s), _p(z), _p(gs))
    if rc:
        raise ValueError(f"orc_quantize_act rc={rc}")
    return dict(q=q, s=s, z=z, gsum=gs)


def quant_sym8(v):
    """One vector -> (int8 codes, scale): the symmetric mapping with b = 8."""
    v = _c(v, np.float32)
    q = np.empty(v.shape[0], np.int8)
    S = ctypes.c_float()
    lib().orc_quant_sym8(_p(v), v.shape[0], _p(q), ctypes.byref(S))
    return q, np.float32(S.value)


def quantize_rows8(X_f16):
    """float16 [M, K] -> dict(q int8 [M,K], s f32 [M]): row-wise INT8 (tokens, or weight channels)."""
    X = _c(X_f16, np.float16)
    M, K = X.shape
    q = np.empty((M, K), np.int8)
    s = np.empty(M, np.float32)
    rc = lib().orc_quantize_rows8(_p(X.view(np.uint16)), M, K, K, _p(q), _p(s))
    if rc:
        raise ValueError(f"orc_quantize_rows8 rc={rc}")
    return dict(q=q, s=s)


def gemm8_i32(A8, W8):
    A, W = _c(A8, np.int8), _c(W8, np.int8)
    M, K = A.shape
    N = W.shape[0]
    P = np.empty((M, N), np.int32)
    rc = lib().orc_gemm8_i32(_p(A), K, _p(W), M, N, K, _p(P))
    if rc:
        raise ValueError(f"orc_gemm8_i32 rc={rc}")
    return P


def linear8(a, w, bias_f16=None, act=ACT_NONE):
    """W8A8 linear: int8 GEMM, then the symmetric per-channel dequantize / bias / GELU / fp16 store of the
    INT4 path (same C routine).  a, w: dicts from quantize_rows8.  Returns dict(P, y f32, out f16)."""
    P = gemm8_i32(a["q"], w["q"])
    M, N = P.shape
    y = dequant(P.reshape(1, M, N), SYM, a["s"], w["s"], bias_f16=bias_f16, act=act)
    return dict(P=P, y=y, out=store_f16(y))


def layernorm_quantize(X_f16, R_f16, gamma_f16, beta_f16, eps, mode=SYM, group=0):
    """LayerNorm(x + r) * gamma + beta per token, then the token-wise quantize of the fp32 result.
    Returns dict(y16 f16 [M,K], y32 f32 [M,K], q, s, z, gsum)."""
    X = _c(X_f16, np.float16)
    M, K = X.shape
    R = None if R_f16 is None else _c(R_f16, np.float16)
    g, b = _c(gamma_f16, np.float16), _c(beta_f16, np.float16)
    assert g.shape == (K,) and b.shape == (K,) and (R is None or R.shape == X.shape)
    ng = _ng(K, group)
    y16 = np.empty((M, K), np.float16)
    y32 = np.empty((M, K), np.float32)
    q = np.empty((M, K // 2), np.uint8)
    s = np.empty(M, np.float32)
    z = np.zeros(M, np.float32)
    gs = np.empty((M, ng), np.int32)
    L = lib()
    L.orc_layernorm_quantize.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p]
    rc = L.orc_layernorm_quantize(_p(X.view(np.uint16)), None if R is None else _p(R.view(np.uint16)), M, K, K,
                                  _p(g.view(np.uint16)), _p(b.view(np.uint16)), float(eps), mode, group,
                                  _p(y16.view(np.uint16)), _p(y32), _p(q), _p(s), _p(z), _p(gs))
    if rc:
        raise ValueError(f"orc_layernorm_quantize rc={rc}")
    return dict(y16=y16, y32=y32, q=q, s=s, z=z, gsum=gs)


def quantize_rows_f32(Y, mode=SYM, group=0):
    Y = _c(Y, np.float32)
    M, K = Y.shape
    ng = _ng(K, group)
    q = np.empty((M, K // 2), np.uint8)
    s = np.empty(M, np.float32)
    z = np.zeros(M, np.float32)
    gs = np.empty((M, ng), np.int32)
    rc = lib().orc_quantize_rows_f32(_p(Y), M, K, K, mode, group, _p(q), _p(s), _p(z), _p(gs))
    if rc:
        raise ValueError(f"orc_quantize_rows_f32 rc={rc}")
    return dict(q=q, s=s, z=z, gsum=gs)


def quantize_weight(W_f16, mode=SYM, group=0):
    """W_f16: float16 [N, K] -> dict(q [N,K/2], s [N,ng], z [N,ng], gsum [N,ng], c [N])."""
    W = _c(W_f16, np.float16)
    N, K = W.shape
    ng = _ng(K, group)
    q = np.empty((N, K // 2), np.uint8)
    s = np.empty((N, ng), np.float32)
    z = np.empty((N, ng), np.float32)
    gs = np.empty((N, ng), np.int32)
    c = np.empty(N, np.float32)
    rc = lib().orc_quantize_weight(_p(W.view(np.uint16)), N, K, mode, group, _p(q), _p(s), _p(z), _p(gs), _p(c))
    if rc:
        raise ValueError(f"orc_quantize_weight rc={rc}")
    return dict(q=q, s=s, z=z, gsum=gs, c=c)


def gemm_i32(Aq, Wq, mode=SYM, group=0, lda=None, K=None):
    """Aq u8 [M, >=K/2] (row stride lda bytes), Wq u8 [N, K/2] -> P i32 [ng, M, N]."""
    Wq = _c(Wq, np.uint8)
    N = Wq.shape[0]
    K = Wq.shape[1] * 2 if K is None else K
    Aq = np.ascontiguousarray(Aq, np.uint8)
    M = Aq.shape[0]
    lda = Aq.shape[1] if lda is None else lda
    ng = _ng(K, group)
    P = np.empty((ng, M, N), np.int32)
    rc = lib().orc_gemm_i32(_p(Aq), lda, _p(Wq), M, N, K, mode, group, _p(P))
    if rc:
        raise ValueError(f"orc_gemm_i32 rc={rc}")
    return P


def dequant(P, mode, sa, sw, za=None, RA=None, zw=None, c=None, bias_f16=None, act=ACT_NONE):
    """P i32 [ng, M, N] -> Y f32 [M, N] (scales, zero-point terms, bias, GELU)."""
    P = _c(P, np.int32)
    ng, M, N = P.shape
    sa = _c(sa, np.float32)
    sw = _c(sw, np.float32)
    za = None if za is None else _c(za, np.float32)
    RA = None if RA is None else _c(RA, np.int32)
    zw = None if zw is None else _c(zw, np.float32)
    c = None if c is None else _c(c, np.float32)
    b = None if bias_f16 is None else _c(bias_f16, np.float16).view(np.uint16)
    Y = np.empty((M, N), np.float32)
    rc = lib().orc_dequant(_p(P), M, N, ng, mode, _p(sa), _p(za), _p(RA), _p(sw), _p(zw), _p(c), _p(b), act, _p(Y))
    if rc:
        raise ValueError(f"orc_dequant rc={rc}")
    return Y


def store_f16(Y):
    Y = _c(Y, np.float32)
    out = np.empty(Y.shape, np.uint16)
    lib().orc_store_f16(_p(Y), ctypes.c_size_t(Y.size), _p(out))
    return out.view(np.float16)


def linear(A, W, mode=SYM, group=0, bias_f16=None, act=ACT_NONE,
           requant=False, requant_mode=SYM, requant_group=0, lda=None, K=None):
    """The whole layer on quantized operands.

    A: dict from quantize_act (q, s, z, gsum);  W: dict from quantize_weight.
    Returns dict(y f32 [M,N], and either out f16 [M,N] or q/s/z/gsum of the requantized rows).
    """
    Wq = _c(W["q"], np.uint8)
    N = Wq.shape[0]
    K = Wq.shape[1] * 2 if K is None else K
    Aq = np.ascontiguousarray(A["q"], np.uint8)
    M = Aq.shape[0]
    lda = Aq.shape[1] if lda is None else lda
    _ng(K, group)
    sa = _c(A["s"], np.float32)
    za = _c(A["z"], np.float32) if mode == ASYM else None
    RA = _c(A["gsum"], np.int32) if mode == ASYM else None
    sw = _c(W["s"], np.float32)
    zw = _c(W["z"], np.float32) if mode == ASYM else None
    c = _c(W["c"], np.float32) if mode == ASYM else None
    b = None if bias_f16 is None else _c(bias_f16, np.float16).view(np.uint16)
    y = np.empty((M, N), np.float32)
    res = dict(y=y)
    out16 = oq = os_ = oz = og = None
    if requant:
        rng = _ng(N, requant_group)
        oq = np.empty((M, N // 2), np.uint8)
        os_ = np.empty(M, np.float32)
        oz = np.zeros(M, np.float32)
        og = np.empty((M, rng), np.int32)
        res.update(q=oq, s=os_, z=oz, gsum=og)
    else:
        out16 = np.empty((M, N), np.uint16)
    rc = lib().orc_linear(_p(Aq), lda, _p(sa), _p(za), _p(RA), _p(Wq), _p(sw), _p(zw), _p(c),
                          M, N, K, mode, group, _p(b), act,
                          int(bool(requant)), requant_mode, requant_group,
                          _p(out16), _p(oq), _p(os_), _p(oz), _p(og), _p(y))
    if rc:
        raise ValueError(f"orc_linear rc={rc}")
    if not requant:
        res["out"] = out16.view(np.float16)
    return res


# ------------------------------------------------------------------ fp64 yardstick
def _expand(per_group, R, K):
    a = np.asarray(per_group, np.float64).reshape(R, -1)
    return np.repeat(a, K // a.shape[1], axis=1)


def dequantize_operand(q_packed, mode, scale, zero=None):
    """codes*scale (+zero) in float64; scale/zero are per row [R] or per (row, group) [R, ng]."""
    codes = unpack(q_packed, mode).astype(np.float64)
    R, K = codes.shape
    out = codes * _expand(scale, R, K)
    if mode == ASYM:
        out = out + _expand(zero, R, K)
    return out


def truth64(A, W, mode=SYM, bias_f16=None, act=ACT_NONE):
    """sum_k x^[m,k] w^[n,k] (+bias, GELU) in float64 from the dequantized operands."""
    xh = dequantize_operand(A["q"], mode, A["s"], A.get("z"))
    wh = dequantize_operand(W["q"], mode, W["s"], W.get("z"))
    y = xh @ wh.T
    if bias_f16 is not None:
        y = y + np.asarray(bias_f16, np.float64)[None, :]
    if act == ACT_GELU:
        erf = np.vectorize(math.erf)
        y = 0.5 * y * (1.0 + erf(y / math.sqrt(2.0)))
    return y


# ------------------------------------------------------------------ per-part strategy (Sec. 4.2 / 4.3)
# The four linear parts are separate components whose INT4 quantization can be switched on or off;
# a part that is off runs in the INT8 sibling.  A strategy is a bit set (bit p = part p in INT4),
# plus FUSED_FFN when FFN1 hands requantized codes straight to FFN2 (Sec. 4.2: quantize fused
# behind bias-add / GELU).
PART_QKV, PART_ATTN_OUT, PART_FFN1, PART_FFN2 = range(4)
FUSED_FFN = 16


def strategy_valid(strategy: int) -> bool:
    if strategy < 0 or strategy > 31:
        return False
    both = (1 << PART_FFN1) | (1 << PART_FFN2)
    return not (strategy & FUSED_FFN) or (strategy & both) == both


def strategy_cost(part_us, ffn_fused_us, strategy: int) -> float:
    """Total cost of one strategy: part_us[p][0] = INT8, part_us[p][1] = INT4 for the part alone;
    the fused FFN pair costs ffn_fused_us in place of its two parts."""
    if not strategy_valid(strategy):
        raise ValueError("invalid strategy")
    bit = lambda p: (strategy >> p) & 1
    total = float(part_us[PART_QKV][bit(PART_QKV)]) + float(part_us[PART_ATTN_OUT][bit(PART_ATTN_OUT)])
    if strategy & FUSED_FFN:
        total += float(ffn_fused_us)
    else:
        total += float(part_us[PART_FFN1][bit(PART_FFN1)]) + float(part_us[PART_FFN2][bit(PART_FFN2)])
    return total


def pick_strategy(part_us, ffn_fused_us) -> int:
    """Every valid strategy priced; the cheapest wins, ties go to more INT4 parts, then to the fused pair."""
    best = None
    for s in range(32):
        if not strategy_valid(s):
            continue
        key = (strategy_cost(part_us, ffn_fused_us, s), -bin(s & 15).count("1"), -(s >> 4))
        if best is None or key < best[0]:
            best = (key, s)
    return best[1]


def part_linear(X_f16, W_f16, int4: bool, bias_f16=None, act=ACT_NONE, mode=SYM, group=0):
    """One part, fp16 in, fp16 out: token-wise quantize + linear in INT4 (Sec. 3.1 with b = 4) or in INT8."""
    if int4:
        return linear(quantize_act(X_f16, mode, group), quantize_weight(W_f16, mode, group), mode, group,
                      bias_f16=bias_f16, act=act)["out"]
    return linear8(quantize_rows8(X_f16), quantize_rows8(W_f16), bias_f16=bias_f16, act=act)["out"]


def ffn(X_f16, W1_f16, b1_f16, act1, W2_f16, b2_f16, strategy: int):
    """FFN1 (+ activation) then FFN2 under a strategy (symmetric per-channel weights).  Fused: FFN1's fp32
    outputs are quantized per token without the fp16 rounding in between."""
    if not strategy_valid(strategy):
        raise ValueError("invalid strategy")
    i1, i2 = bool(strategy >> PART_FFN1 & 1), bool(strategy >> PART_FFN2 & 1)
    if strategy & FUSED_FFN:
        H = linear(quantize_act(X_f16), quantize_weight(W1_f16), bias_f16=b1_f16, act=act1, requant=True)
        return linear(H, quantize_weight(W2_f16), bias_f16=b2_f16)["out"]
    H16 = part_linear(X_f16, W1_f16, i1, b1_f16, act1)
    return part_linear(H16, W2_f16, i2, b2_f16)


# ------------------------------------------------------------------ whole encoder layer (Sec. 4.2: the pipeline
# around the four linears: FP16 attention between QKV and the output projection, LayerNorm (+ residual) after
# the attention output and after the MLP)
FUSED_LN = 32


def attention(QKV_f16, batch: int, seq: int, heads: int):
    """softmax(Q K^T / sqrt(d)) V per sequence and head, in float64.  QKV_f16 [batch*seq, 3h]: columns [0,h) are
    the queries, [h,2h) the keys, [2h,3h) the values; head j owns columns j*d .. (j+1)*d of each.  No mask.
    Returns float64 [batch*seq, h]."""
    QKV = np.asarray(QKV_f16, np.float16).astype(np.float64)
    M, h3 = QKV.shape
    h = h3 // 3
    d = h // heads
    assert M == batch * seq and h * 3 == h3 and d * heads == h
    out = np.empty((M, h), np.float64)
    for b in range(batch):
        rows = slice(b * seq, (b + 1) * seq)
        for j in range(heads):
            q = QKV[rows, j * d:(j + 1) * d]
            k = QKV[rows, h + j * d:h + (j + 1) * d]
            v = QKV[rows, 2 * h + j * d:2 * h + (j + 1) * d]
            s = (q @ k.T) / math.sqrt(d)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=1, keepdims=True)
            out[rows, j * d:(j + 1) * d] = p @ v
    return out


def encoder_layer(X_f16, batch, seq, heads, Wqkv, bqkv, Wao, bao, W1, b1, W2, b2, g1, be1, g2, be2, eps, strategy):
    """One post-LayerNorm encoder layer, fp16 in, fp16 out (symmetric per-channel weights):
        x1  = LN1(x + attn_out(attention(qkv(x))));   out = LN2(x1 + ffn2(gelu(ffn1(x1))))
    Strategy bits as for pick_strategy; FUSED_LN: FFN1 consumes the codes LN1 produced from its fp32 result
    (Sec. 4.2: quantize fused with the LayerNorm) instead of quantizing the fp16 copy of x1."""
    X = np.asarray(X_f16, np.float16)
    bit = lambda p: bool(strategy >> p & 1)
    if strategy & FUSED_LN and not bit(PART_FFN1):
        raise ValueError("FUSED_LN needs FFN1 in INT4")
    qkv = part_linear(X, Wqkv, bit(PART_QKV), bqkv)
    ctx = store_f16(attention(qkv, batch, seq, heads).astype(np.float32))
    ao = part_linear(ctx, Wao, bit(PART_ATTN_OUT), bao)
    ln1 = layernorm_quantize(ao, X, g1, be1, eps)
    x1 = ln1["y16"]
    if strategy & FUSED_LN:
        if strategy & FUSED_FFN:
            H = linear(ln1, quantize_weight(W1), bias_f16=b1, act=ACT_GELU, requant=True)
            h2 = linear(H, quantize_weight(W2), bias_f16=b2)["out"]
        else:
            H16 = linear(ln1, quantize_weight(W1), bias_f16=b1, act=ACT_GELU)["out"]
            h2 = part_linear(H16, W2, bit(PART_FFN2), b2)
    else:
        h2 = ffn(x1, W1, b1, ACT_GELU, W2, b2, strategy & 31)
    return layernorm_quantize(h2, x1, g2, be2, eps)["y16"]
