"""The FP16 attention stand-in and the whole encoder layer (Sec. 4.2: FP16 attention between the quantized
linears, LayerNorm after the attention output and the MLP, the launch sequence replayed from a graph for small
inputs): against the oracle, against the entry points the layer is composed of, and under graph replay."""
import numpy as np
import pytest
import torch

from tests.gpu_util import dev, has_gpu, host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not has_gpu(), reason="needs a GPU")]


@pytest.fixture(scope="module")
def B():
    from paper_2301_12017_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("batch,seq,heads", [(1, 128, 12), (3, 37, 2), (2, 512, 1), (5, 1, 3), (1, 70, 16)])
def test_attention_against_the_oracle(B, orc, batch, seq, heads):
    rng = np.random.default_rng(batch + seq + heads)
    QKV = (rng.standard_normal((batch * seq, 3 * heads * 64)) * 1.5).astype(np.float16)
    got = host(B.attention(dev(QKV), batch, seq, heads)).astype(np.float64)
    want = orc.attention(QKV, batch, seq, heads)
    # fp32 sums of <= 512 terms and one fp16 rounding of the result
    assert np.abs(got - want).max() <= 1e-3 * np.abs(want) .max() + 1e-3 * np.sqrt((want ** 2).mean())
    np.testing.assert_allclose(got, want, rtol=2e-3, atol=2e-3 * np.sqrt((want ** 2).mean()))


def test_attention_of_peaked_scores_does_not_overflow(B, orc):
    batch, seq, heads = 1, 64, 2
    rng = np.random.default_rng(3)
    QKV = (rng.standard_normal((seq, 3 * heads * 64)) * 12).astype(np.float16)      # scores of a few hundred
    got = host(B.attention(dev(QKV), batch, seq, heads)).astype(np.float64)
    want = orc.attention(QKV, batch, seq, heads)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, want, rtol=3e-3, atol=3e-2)


def _layer(B, seed, batch, seq, heads, h, f, layout=None):
    rng = np.random.default_rng(seed)
    n = lambda *s, std=1.0: (rng.standard_normal(s) * std).astype(np.float16)
    t = dict(X=n(batch * seq, h), Wqkv=n(3 * h, h, std=0.05), bqkv=n(3 * h, std=0.02), Wao=n(h, h, std=0.05),
             bao=n(h, std=0.02), W1=n(f, h, std=0.05), b1=n(f, std=0.02), W2=n(h, f, std=0.05), b2=n(h, std=0.02),
             g1=(1 + 0.1 * rng.standard_normal(h)).astype(np.float16), be1=n(h, std=0.1),
             g2=(1 + 0.1 * rng.standard_normal(h)).astype(np.float16), be2=n(h, std=0.1))
    d = {k: dev(v) for k, v in t.items()}
    L = B.EncoderLayer(batch, seq, heads, d["Wqkv"], d["bqkv"], d["Wao"], d["bao"], d["W1"], d["b1"], d["W2"], d["b2"],
                       d["g1"], d["be1"], d["g2"], d["be2"], 1e-12, layout=layout)
    return t, d, L


def _blocks(B, L, d, strategy):
    """The layer spelled out with the entry points it is made of."""
    X = d["X"]
    M, h = X.shape
    qkv = B.part_linear(X, L.qkv, bool(strategy & 1))
    ctx = B.attention(qkv, L.batch, L.seq, L.heads)
    ao = B.part_linear(ctx, L.attn_out, bool(strategy & 2))
    a1 = B._new_qact(M, h, B.SYM, 0, L.ffn1.w4.layout, X.device)
    x1 = torch.empty_like(X)
    B.layernorm_quantize(ao, X, d["g1"], d["be1"], 1e-12, out=a1, y=x1, layout=L.ffn1.w4.layout)
    if strategy & B.STRATEGY_FUSED_LN:
        if strategy & B.STRATEGY_FUSED_FFN:
            H = B.linear(a1, L.ffn1.w4, d["b1"], B.ACT_GELU, requant=True, requant_layout=L.ffn2.w4.layout)
            h2 = B.linear(H, L.ffn2.w4, d["b2"])
        else:
            H = B.linear(a1, L.ffn1.w4, d["b1"], B.ACT_GELU)
            h2 = B.part_linear(H, L.ffn2, bool(strategy & 8))
    else:
        h2 = B.ffn(x1, L.ffn1, L.ffn2, strategy & 31)
    a2 = B._new_qact(M, h, B.SYM, 0, 0, X.device)
    out = torch.empty_like(X)
    B.layernorm_quantize(h2, x1, d["g2"], d["be2"], 1e-12, out=a2, y=out)
    return out


STRATEGIES = [0, 4, 15, 15 | 32, 31, 31 | 32, 7 | 32]


@pytest.mark.parametrize("shape", [(1, 128, 12, 768, 3072), (16, 128, 4, 256, 1024), (3, 21, 2, 128, 256)])
@pytest.mark.parametrize("strategy", STRATEGIES)
def test_layer_equals_its_building_blocks(B, shape, strategy):
    batch, seq, heads, h, f = shape
    t, d, L = _layer(B, sum(shape), batch, seq, heads, h, f)
    got = L(d["X"], strategy)
    assert torch.equal(got, _blocks(B, L, d, strategy))
    assert torch.isfinite(got.float()).all()


@pytest.mark.parametrize("strategy", STRATEGIES)
def test_layer_against_the_oracle(B, orc, strategy):
    batch, seq, heads, h, f = 2, 24, 2, 128, 256
    t, d, L = _layer(B, 77, batch, seq, heads, h, f)
    got = host(L(d["X"], strategy)).astype(np.float64)
    want = orc.encoder_layer(t["X"], batch, seq, heads, t["Wqkv"], t["bqkv"], t["Wao"], t["bao"], t["W1"], t["b1"], t["W2"],
                             t["b2"], t["g1"], t["be1"], t["g2"], t["be2"], 1e-12, strategy).astype(np.float64)
    # last-bit differences of the attention / GELU / LayerNorm values move a few INT4 codes of the next part
    # by one step, so whole-layer agreement is statistical; the pieces are checked one by one elsewhere
    rms = np.sqrt((want ** 2).mean())
    assert np.sqrt(((got - want) ** 2).mean()) < 1e-2 * rms
    assert np.abs(got - want).max() < 0.25 * rms


def test_layer_replays_from_a_graph(B):
    """The b1/s128 BERT-base layer captured once and replayed: every replay equals the eager result, with
    eager work of the same library (which shares no buffer with the graph) in between."""
    batch, seq, heads, h, f = 1, 128, 12, 768, 3072
    t, d, L = _layer(B, 5, batch, seq, heads, h, f)
    _, d2, L2 = _layer(B, 6, batch, seq, heads, h, f)
    for strategy in (15, 31 | 32):
        eager = L(d["X"], strategy).clone()
        out = torch.empty_like(eager)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            L(d["X"], strategy, out=out, stream=side.cuda_stream)              # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            L(d["X"], strategy, out=out, stream=side.cuda_stream)
        for rep in range(4):
            out.zero_()
            other = L2(d2["X"], strategy)                                        # eager work between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), (strategy, rep)
            assert torch.isfinite(other.float()).all()


@pytest.mark.parametrize("shape", [(1, 128, 12, 768, 3072), (5, 100, 8, 512, 1024)])
@pytest.mark.parametrize("strategy", STRATEGIES)
def test_layer_with_weights_in_the_fp6_layout(B, shape, strategy):
    """Every INT4 part on the FP6 matrix instruction (LayerNorm writes the FP6 operand, the fused FFN pair hands FP6 codes
    over): the layer equals the entry points it is made of, and - the FP6 kernels and the canonical-layout kernels both
    follow the definition's operation order - the same layer with canonical weights, bit for bit."""
    batch, seq, heads, h, f = shape
    t, d, L6 = _layer(B, sum(shape), batch, seq, heads, h, f, layout=B.LAYOUT_FP6)
    got = L6(d["X"], strategy)
    assert torch.equal(got, _blocks(B, L6, d, strategy))
    _, _, L0 = _layer(B, sum(shape), batch, seq, heads, h, f, layout=B.LAYOUT_CANONICAL)
    assert torch.equal(got, L0(d["X"], strategy))
    assert B.fused_fault_check() is False
