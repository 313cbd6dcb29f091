"""Seeded synthetic inputs for the W4A4 linear layer, shared by the tests, the
smoke check and the benchmark.

This module holds no arithmetic of the method: it only draws fp16 tensors with
the shapes of the encoder linears (Sec. 4.1: (bs*seq) x {3h, h, 4h, h} x
{h, h, h, 4h}) and the value distributions the workloads fix.  The same bits
are handed to the CPU oracle and uploaded to the GPU.

All draws come from numpy's PCG64 seeded with SeedSequence([seed, config,
tensor_id]) as float32 standard normals, scaled, then rounded to float16.
"""
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

SYM, ASYM = 0, 1


@dataclass(frozen=True)
class LinearSpec:
    name: str
    M: int
    N: int
    K: int
    gelu: bool = False
    mode: int = SYM
    group: int = 0          # 0 = one weight scale per output channel


def _encoder_linears(M: int, h: int, ffn: int, mode=SYM, group=0) -> List[LinearSpec]:
    return [
        LinearSpec("qkv", M, 3 * h, h, False, mode, group),
        LinearSpec("attn_out", M, h, h, False, mode, group),
        LinearSpec("ffn1", M, ffn, h, True, mode, group),
        LinearSpec("ffn2", M, h, ffn, False, mode, group),
    ]


def config_linears(cfg: int) -> List[LinearSpec]:
    """The GEMM list of workload `cfg` (1-based, in the order the baseline file lists them)."""
    if cfg == 1:
        return [LinearSpec("single", 128, 768, 768)]
    if cfg == 2:
        return _encoder_linears(128, 768, 3072)
    if cfg == 3:
        return _encoder_linears(12288, 1024, 4096)
    if cfg == 4:
        return _encoder_linears(16384, 768, 3072, ASYM, 128)
    if cfg == 5:
        return _encoder_linears(32768, 1024, 4096)
    raise ValueError(cfg)


def _rng(seed: int, cfg: int, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, cfg, tensor_id]))


def normal_f16(shape, std: float, seed: int, cfg: int, tensor_id: int) -> np.ndarray:
    x = _rng(seed, cfg, tensor_id).standard_normal(shape, dtype=np.float32)
    x *= np.float32(std)
    return x.astype(np.float16)


def activations(M: int, K: int, seed=0, cfg=1, tensor_id=0, outlier_channels: int = 0,
                outlier_gain: float = 20.0) -> np.ndarray:
    """X ~ N(0,1) as fp16 [M,K].  With outlier_channels > 0, that many distinct
    hidden channels (the same for every token) are multiplied by outlier_gain,
    imitating the wide activation ranges the paper reports for some models."""
    x = _rng(seed, cfg, tensor_id).standard_normal((M, K), dtype=np.float32)
    if outlier_channels:
        cols = _rng(seed, cfg, 1000 + tensor_id).choice(K, outlier_channels, replace=False)
        x[:, cols] *= np.float32(outlier_gain)
    return x.astype(np.float16)


def weights(N: int, K: int, seed=0, cfg=1, tensor_id=1) -> np.ndarray:
    """W ~ N(0, 0.02) as fp16 [N,K] (row n = output channel n)."""
    return normal_f16((N, K), 0.02, seed, cfg, tensor_id)


def bias(N: int, seed=0, cfg=1, tensor_id=2) -> np.ndarray:
    """b ~ N(0, 0.01) as fp16 [N]."""
    return normal_f16((N,), 0.01, seed, cfg, tensor_id)


def linear_inputs(spec: LinearSpec, cfg: int, index: int, seed: int = 0, M: Optional[int] = None):
    """(X, W, b) for the index-th linear of a workload.  tensor ids: 10*index + {0,1,2}."""
    m = spec.M if M is None else M
    x = activations(m, spec.K, seed, cfg, 10 * index, outlier_channels=8 if cfg == 4 else 0)
    w = weights(spec.N, spec.K, seed, cfg, 10 * index + 1)
    b = bias(spec.N, seed, cfg, 10 * index + 2)
    return x, w, b
