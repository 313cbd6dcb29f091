"""Helpers shared by the GPU parity tests: host<->device copies and oracle views."""
import numpy as np
import torch


def has_gpu():
    return torch.cuda.is_available()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return None if t is None else t.detach().cpu().numpy()


def act_to_canonical(q, mode=0):
    """Bytes of activations in the MFMA operand layout -> canonical bytes.  Symmetric codes: the low nibble is
    offset binary (flip its top bit); unsigned codes: the high nibble holds u - 8 (flip ITS top bit).
    A pure re-encoding; no arithmetic of the method."""
    return q ^ np.uint8(0x08 if mode == 0 else 0x80)


def wgt_to_canonical(q, mode=0):
    """Bytes of weights in the MFMA operand layout -> canonical bytes: the nibbles are swapped; symmetric codes
    keep the odd element (low nibble) in offset binary, unsigned codes the even element (high nibble) as u - 8."""
    if mode == 0:
        return ((q >> 4) | (((q & 0x0F) ^ 0x08) << 4)).astype(np.uint8)
    return (((q >> 4) ^ 0x08) | ((q & 0x0F) << 4)).astype(np.uint8)


def qact_host(A):
    """QAct (device) -> the dict layout the oracle uses (codes in the canonical packing)."""
    q = host(A.q)
    d = dict(q=act_to_canonical(q, A.mode) if getattr(A, "layout", 0) == 1 else q, s=host(A.scale))
    d["z"] = host(A.zero) if A.zero is not None else np.zeros(A.M, np.float32)
    d["gsum"] = host(A.gsum) if A.gsum is not None else None
    return d


def qweight_host(W):
    q = host(W.q)
    d = dict(q=wgt_to_canonical(q, W.mode) if getattr(W, "layout", 0) == 1 else q, s=host(W.scale),
             gsum=host(W.gsum), c=host(W.rowsum_deq))
    d["z"] = host(W.zero) if W.zero is not None else np.zeros_like(d["s"])
    return d


def f16_close(got_f16, want_f16, want_f32=None):
    """The acceptance bar for fp16 outputs: |gpu - oracle| <= 1e-2*|oracle| + 1e-3*rms(oracle).
    (1e-2 relative is the stated target; the absolute floor covers GELU's negative tail and fp16
    subnormals, where a relative bound is meaningless.)  Returns (ok, max_violation_ratio)."""
    g = got_f16.astype(np.float64)
    w = want_f16.astype(np.float64)
    fin = np.isfinite(w)
    if not np.array_equal(np.isfinite(g), fin):
        return False, np.inf
    rms = np.sqrt(np.mean(w[fin] ** 2)) if fin.any() else 0.0
    tol = 1e-2 * np.abs(w[fin]) + 1e-3 * rms
    err = np.abs(g[fin] - w[fin])
    ratio = float(np.max(err / np.maximum(tol, 1e-300))) if err.size else 0.0
    return ratio <= 1.0, ratio


# Bars for fp16 outputs beyond the tolerance of f16_close (fractions of bit-identical values; the rest may be one
# fp16 step off):
#   GELU stores: the device evaluates the erf form with a degree-5 tail to fp16 accuracy (relative error < 9e-5):
#     one step at most, about 95 % of the values identical to the oracle's;
#   the persistent operand-layout kernel without GELU: the same real number as the definition, evaluated with
#     fused multiply-adds (a few fp32 units in the last place apart): identical except on near-ties of the fp16 grid.
GELU_SAME = 0.92
OLAY_SAME = 0.995


def f16_steps(got, want):
    """(fraction of bit-identical values, largest distance in steps of the fp16 grid); -0 and +0 coincide."""
    def key(a):
        u = np.ascontiguousarray(a).view(np.uint16).astype(np.int64)
        return np.where(u & 0x8000, -(u & 0x7FFF), u)
    d = np.abs(key(got) - key(want))
    return (float(np.mean(d == 0)), int(d.max())) if d.size else (1.0, 0)


def assert_f16(got, want, min_same, what=""):
    """At least `min_same` of the values identical (1.0: bit for bit), the rest at most one fp16 step apart --
    or, for values that cancel to (almost) nothing, within 4e-6 of the rms output, where a step of the fp16
    grid is smaller than the fp32 rounding noise of the terms that cancel."""
    if min_same >= 1.0:
        assert np.array_equal(np.ascontiguousarray(got).view(np.uint16), np.ascontiguousarray(want).view(np.uint16)), what
        return
    def key(a):
        u = np.ascontiguousarray(a).view(np.uint16).astype(np.int64)
        return np.where(u & 0x8000, -(u & 0x7FFF), u)
    steps = np.abs(key(got) - key(want))
    g, w = got.astype(np.float64), want.astype(np.float64)
    tiny = np.abs(g - w) <= 2.0 ** -18 * np.sqrt(np.mean(w ** 2))
    same = float(np.mean(steps == 0))
    assert np.all((steps <= 1) | tiny) and same >= min_same, f"{what}: {same:.5f} identical, {int(steps[~tiny].max(initial=0))} steps"


def asym_budget(orc, a, w, group):
    """fp32 rounding noise that ANY evaluation order of the unsigned mapping's dequantize carries, per output element:
    y = sa*sum_g sw*P_g + sa*sum_g zw*RA + za*c + b is a small difference of large terms (with outlier channels
    |sa*t1| is hundreds of times |y|), and every one of the ng + 4 roundings on the way costs up to half a unit in
    the last place of those terms.  Two faithful fp32 evaluations (the oracle's order, a kernel's fused order) can
    differ by twice that.  a, w: the oracle-style dicts of the (sampled) activations and of the weights."""
    K = a["q"].shape[1] * 2
    G = K if group == 0 else group
    ng = K // G
    P = orc.gemm_i32(a["q"], w["q"], 1, group).astype(np.float64)              # [ng, M, N]
    sw, zw = w["s"].reshape(-1, ng).astype(np.float64), w["z"].reshape(-1, ng).astype(np.float64)
    ra = a["gsum"].reshape(-1, ng).astype(np.float64)
    sa, za = a["s"].astype(np.float64)[:, None], a["z"].astype(np.float64)[:, None]
    t1 = np.einsum("gmn,ng->mn", np.abs(P), np.abs(sw))
    t2 = np.abs(ra) @ np.abs(zw).T
    mag = np.abs(sa) * (t1 + t2) + np.abs(za) * np.abs(w["c"].astype(np.float64))[None, :]
    return 2.0 * (ng + 4) * 2.0 ** -24 * mag


def f16_close_budget(got_f16, want_f16, budget):
    """f16_close with a per-element absolute allowance added to the tolerance.  Returns (ok, worst ratio)."""
    g, w = got_f16.astype(np.float64), want_f16.astype(np.float64)
    tol = 1e-2 * np.abs(w) + 1e-3 * np.sqrt(np.mean(w ** 2)) + budget
    ratio = float(np.max(np.abs(g - w) / tol))
    return ratio <= 1.0, ratio


def olay_schedules(B, K):
    """Schedule numbers of the persistent operand-layout kernel (every tile shape takes any K % 128 == 0, K >= 256)."""
    assert K % 128 == 0 and K >= 256
    return [i + 1 for i, n in enumerate(B.schedule_names()) if n.startswith("olay")]


# ---- the FP6 operand layout (a re-encoding of the codes; no arithmetic of the method) -------------------------------
_FP6_VALUE = {0: 0, 8: 1, 16: 2, 20: 3, 24: 4, 26: 5, 28: 6, 30: 7}     # E2M3 magnitude field -> integer it encodes


def fp6_plan(K):
    """(lanes per row, operands per lane) of the token-wise quantizer of the FP6 layout, or None for a K the layout is not
    offered for: the fewest lanes (8, 16, 32, 64; a divisor of K/32) that keep the operands per lane <= 2, else <= 3, 4, 6."""
    n_op = K // 32
    if K % 64 or K > 10240:
        return None
    for most in (2, 3, 4, 6):
        for lpr in (8, 16, 32, 64):
            if n_op % lpr == 0 and n_op // lpr <= most:
                return lpr, n_op // lpr
    return None


def fp6_to_codes(q, K, rows, weight=False):
    """A matrix in the FP6 operand layout -> int8 codes [rows, K] in the order of K.
    Rows come in panels (64 tokens; 128 channels, channel n in storage row (n % 4) * 32 + (n % 128) / 4); a panel is
    K/64 blocks of [rows of the panel][48 bytes]; operand 2b + h of a row lies in its 48 bytes of block b as 16 bytes
    at 16h and 8 bytes at 32 + 8h (at 40 - 8h in storage rows 16 .. 31 of every 32); its 32 six-bit fields (little-endian) hold
    codes 32o .. 32o+31 of the row, for operand index o.  Padding rows must be zeros (of either sign)."""
    R = 128 if weight else 64
    n_op, kb = K // 32, K // 64
    flat = np.ascontiguousarray(q).reshape(-1)
    padded = (rows + R - 1) // R * R
    assert flat.size == padded * K // 4 * 3
    blocks = flat.reshape(padded // R, kb, R, 48)                                # [panel, block, storage row, 48]
    r = np.arange(padded)
    srow = ((r % 4) * 32 + (r % 128) // 4) if weight else (r % 64)
    blocks = blocks[r // R, :, srow, :]                                          # [row, block, 48]
    ops = np.empty((padded, n_op, 24), np.uint8)
    swap = ((srow >> 4) & 1).astype(bool)                                        # storage rows 16 .. 31 of every 32: 8-byte parts exchanged
    for h in (0, 1):
        ops[:, h::2, :16] = blocks[:, :, 16 * h:16 * h + 16]
        ops[:, h::2, 16:] = np.where(swap[:, None, None], blocks[:, :, 40 - 8 * h:48 - 8 * h], blocks[:, :, 32 + 8 * h:40 + 8 * h])
    bits = np.unpackbits(ops, axis=2, bitorder="little").reshape(padded, n_op, 32, 6)
    fields = (bits * (1 << np.arange(6, dtype=np.int64))).sum(axis=3)            # [padded rows, n_op, 32]
    # padding rows hold zeros; a fused epilogue may write them as negative zeros (the sign bit of a field set)
    assert not (fields[rows:] & 31).any(), "padding rows are not zero"
    fields = fields[:rows]
    mag = fields & 31
    assert np.isin(mag, list(_FP6_VALUE)).all(), "a field that is not an integer of magnitude <= 7"
    lut = np.zeros(32, np.int64)
    for k_, v_ in _FP6_VALUE.items():
        lut[k_] = v_
    val = np.where(fields & 32, -lut[mag], lut[mag])
    return val.reshape(rows, K).astype(np.int8)                                   # operand o, field f: code 32 o + f


def fp6_schedules(B, K):
    """Schedule numbers of the FP6 kernels that take this K (the seven-stage ring of the 192 x 256 tile wants at least
    nine half steps of 64 codes)."""
    return [i + 1 for i, n in enumerate(B.schedule_names()) if n.startswith("fp6") and not (n == "fp6_192x256" and K < 640)]
