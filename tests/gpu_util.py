"""Helpers shared by the GPU parity tests: host<->device copies and oracle views."""
import numpy as np
import torch


def has_gpu():
    return torch.cuda.is_available()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return None if t is None else t.detach().cpu().numpy()


def act_to_canonical(q):
    """Bytes of activations in the MFMA operand layout -> canonical bytes (the low nibble is
    offset binary: flip its top bit).  A pure re-encoding; no arithmetic of the method."""
    return q ^ np.uint8(0x08)


def wgt_to_canonical(q):
    """Bytes of weights in the MFMA operand layout -> canonical bytes (the nibbles are swapped
    and the low one, the odd element, is offset binary)."""
    return ((q >> 4) | (((q & 0x0F) ^ 0x08) << 4)).astype(np.uint8)


def qact_host(A):
    """QAct (device) -> the dict layout the oracle uses (codes in the canonical packing)."""
    q = host(A.q)
    d = dict(q=act_to_canonical(q) if getattr(A, "layout", 0) == 1 else q, s=host(A.scale))
    d["z"] = host(A.zero) if A.zero is not None else np.zeros(A.M, np.float32)
    d["gsum"] = host(A.gsum) if A.gsum is not None else None
    return d


def qweight_host(W):
    q = host(W.q)
    d = dict(q=wgt_to_canonical(q) if getattr(W, "layout", 0) == 1 else q, s=host(W.scale),
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


def olay_schedules(B, K):
    """Schedule numbers of the persistent operand-layout kernel (every tile shape takes any K % 128 == 0, K >= 256)."""
    assert K % 128 == 0 and K >= 256
    return [i + 1 for i, n in enumerate(B.schedule_names()) if n.startswith("olay")]
