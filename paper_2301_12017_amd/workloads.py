"""Device-side harness for the synthetic workloads: uploads the seeded tensors, quantizes
the weights once (offline step) and strings the library calls together the way an encoder
layer would (Sec. 4.1 shapes, Sec. 4.2 fusion).  All arithmetic happens in libw4a4.so; this
module only owns tensors and call order.  Used by the tests, the smoke check and bench.py.
"""
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from . import binding as B
from . import synth


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@dataclass
class Layer:
    spec: synth.LinearSpec
    W: B.QWeight
    bias: torch.Tensor
    act: int
    host_W: Optional[np.ndarray] = None
    host_b: Optional[np.ndarray] = None


def make_layer(spec: synth.LinearSpec, cfg: int, index: int, seed: int = 0, keep_host: bool = True,
               layout: Optional[int] = None) -> Layer:
    """Weights of one linear, quantized offline in the layout the library prefers for the shape
    (or the one asked for)."""
    w = synth.weights(spec.N, spec.K, seed, cfg, 10 * index + 1)
    b = synth.bias(spec.N, seed, cfg, 10 * index + 2)
    if layout is None:
        layout = B.preferred_layout(spec.M, spec.N, spec.K, spec.mode, spec.group)
    Wq = B.quantize_weight(dev(w), spec.mode, spec.group, layout=layout)
    return Layer(spec, Wq, dev(b), B.ACT_GELU if spec.gelu else B.ACT_NONE,
                 w if keep_host else None, b if keep_host else None)


def make_input(spec: synth.LinearSpec, cfg: int, index: int, seed: int = 0, M: Optional[int] = None) -> np.ndarray:
    return synth.activations(spec.M if M is None else M, spec.K, seed, cfg, 10 * index,
                             outlier_channels=8 if cfg == 4 else 0)


def run_linear(X: torch.Tensor, layer: Layer, schedule: int = 0, qact: Optional[B.QAct] = None,
               out=None) -> torch.Tensor:
    """quantize_act followed by the fused linear with an fp16 store."""
    A = B.quantize_act(X, layer.spec.mode, layer.spec.group, out=qact, layout=layer.W.layout)
    return B.linear(A, layer.W, layer.bias, layer.act, schedule=schedule, out=out)


# ------------------------------------------------------------------ the chained stack
@dataclass
class ChainLayer:
    qkv: Layer
    out: Layer
    ffn1: Layer
    ffn2: Layer


def make_chain(n_layers: int, h: int = 1024, ffn: int = 4096, M: int = 32768, cfg: int = 5, seed: int = 0,
               keep_host: bool = True, layout: int = B.LAYOUT_CANONICAL) -> List[ChainLayer]:
    layers = []
    for l in range(n_layers):
        specs = [synth.LinearSpec("qkv", M, 3 * h, h), synth.LinearSpec("attn_out", M, h, h),
                 synth.LinearSpec("ffn1", M, ffn, h, True), synth.LinearSpec("ffn2", M, h, ffn)]
        layers.append(ChainLayer(*[make_layer(s, cfg, 4 * l + j, seed, keep_host, layout) for j, s in enumerate(specs)]))
    return layers


def v_slice(qkv: B.QAct, h: int) -> B.QAct:
    """The V third of a requantized QKV output, read in place: columns [2h, 3h) of every
    packed row, i.e. byte offset h, row stride 3h/2, with the QKV output's per-token scale
    (and, in the MFMA operand layout, the third column slice's odd-position sums).  In the FP6 operand layout the
    slice is blocks 2h/64 .. 3h/64 - 1 of every 64-token panel: the pointer moves to the first of them (3072 bytes
    each) and lda keeps the full matrix's value, from which the panel length follows."""
    off = (2 * h // 64) * 3072 if qkv.layout == B.LAYOUT_FP6 else h
    return B.QAct(qkv.q, qkv.scale, qkv.zero, None, qkv.M, h, qkv.lda, 0, qkv.mode, q_offset_bytes=off,
                  layout=qkv.layout, osum=qkv.osum, osum_index=2 if qkv.osum is not None else 0)


def run_chain(A: B.QAct, layers: List[ChainLayer], workspace: Optional[torch.Tensor] = None, record=None,
              schedule: int = 0) -> B.QAct:
    """quantize -> GEMM -> dequant+bias(+GELU) -> requantize, four GEMMs per layer, without
    an fp16 activation tensor in between.  `record` (a list) receives (name, input, output).
    The requantized outputs keep the layout of the operands; the QKV output keeps one
    odd-position sum per third so that the V slice can be consumed in place."""
    h = layers[0].out.spec.K
    for li, L in enumerate(layers):
        steps = (("qkv", L.qkv, None), ("attn_out", L.out, h), ("ffn1", L.ffn1, None), ("ffn2", L.ffn2, None))
        for name, lay, slice_h in steps:
            a_in = v_slice(A, slice_h) if slice_h else A
            mfma = lay.W.layout == B.LAYOUT_MFMA
            out = B.linear(a_in, lay.W, lay.bias, lay.act, requant=True, requant_mode=B.SYM, schedule=schedule,
                           workspace=workspace, requant_layout=lay.W.layout,
                           requant_group=h if (mfma and name == "qkv") else 0)
            if record is not None:
                record.append((li, name, a_in, out, lay))
            A = out
    return A
