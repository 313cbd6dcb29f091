#!/usr/bin/env python3
"""Benchmark of the W4A4 linear hot path on one MI355X.

A step is one pass of the whole path -- token-wise quantize_act, then the fused
INT4 GEMM + dequantize/bias(/GELU) epilogue with an fp16 store -- over the four
encoder linears of BERT-large at batch 32 x seq 384 (M = 12288; Sec. 4.1 shapes),
with fp16 activations, quantized weights and biases already resident in HBM.
`value` is 2*M*N*K summed over the four GEMMs divided by the step time (so the
quantize kernels count against it).  The line also carries the latency of the
BERT-base layer linears at batch 1 x seq 128, the roofline position of the GEMM
kernel (HIP events around every w4a4_linear launch inside the timed region) and the
CPU oracle timed on a sample of token rows of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0      # MI355X dense int8 matrix peak, 5.0 POP/s
HBM_PEAK_GBS = 8000.0
# HBM-side bytes of the four w4a4_linear launches of one step of configs[2], from the rocprofv3 --pmc
# runs summarised in profiles/gemm_config3_hbm_traffic.txt (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the
# factors a 256 MiB device copy gave in the same runs).  Not measured live; None for other workloads.
PROFILED_TRAFFIC_BYTES = {3: int((18.52 + 10.36 + 22.82 + 42.86 + 72.0 + 24.0 + 96.0 + 24.0) * 2 ** 20)}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=50)
    p.add_argument("--warmup", type=int, default=10)
    p.add_argument("--config", type=int, default=3, help="workload number (3 = headline, 4 = asymmetric/grouped, 5 = one layer of the chained stack)")
    p.add_argument("--schedule", type=int, default=0, help="force a GEMM tile schedule (0 = built-in table)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--settle-ms", type=float, default=300.0,
                   help="untimed steps run for this long before the warm-up steps: after an idle phase the chip's "
                        "clocks dip for some milliseconds a few milliseconds into a burst of work, and a short timed "
                        "region that starts right after set-up would measure that transient instead of the sustained rate")
    p.add_argument("--gemm-curve", action="store_true",
                   help="instead of the step: INT4 and INT8 GEMM kernel time over the token count for the BERT-base and "
                        "BERT-large shapes (the comparison of Sec. 4.1 on this hardware); prints its own JSON line")
    p.add_argument("--step-only", action="store_true",
                   help="only the timed step and its roofline: skip the latency, fusion, sibling, strategy and library legs "
                        "(for profiler runs, so that a kernel trace holds the step's launches alone)")
    p.add_argument("--copy-probe-mb", type=int, default=0,
                   help="also run one plain device copy of this many MiB (a kernel of known traffic, used to "
                        "calibrate the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    p.add_argument("--cpu-rows", type=int, default=1024, help="token rows per GEMM the oracle is timed on")
    return p.parse_args()


def settle(fn, ms):
    """Keeps the GPU busy with untimed calls of fn for `ms` milliseconds (checked every ten calls, so that the
    launch queue stays short)."""
    import torch
    t_end = time.perf_counter() + ms * 1e-3
    while time.perf_counter() < t_end:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()


def cpu_baseline(specs, cfg, rows):
    """The oracle as it stands (single thread, plain C) on `rows` token rows of every GEMM."""
    import numpy as np
    import oracle
    from paper_2301_12017_amd import synth
    ops = 0
    prepared = []
    for i, s in enumerate(specs):
        X = synth.activations(rows, s.K, 0, cfg, 10 * i, outlier_channels=8 if cfg == 4 else 0)
        W = synth.weights(s.N, s.K, 0, cfg, 10 * i + 1)
        b = synth.bias(s.N, 0, cfg, 10 * i + 2)
        Q = oracle.quantize_weight(W, s.mode, s.group)            # offline step, not timed
        prepared.append((s, X, Q, b))
        ops += 2 * rows * s.N * s.K
    t0 = time.perf_counter()
    for s, X, Q, b in prepared:
        A = oracle.quantize_act(X, s.mode, s.group)
        oracle.linear(A, Q, s.mode, s.group, b, oracle.ACT_GELU if s.gelu else oracle.ACT_NONE)
    dt = time.perf_counter() - t0
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": 1, "kind": "oracle",
            "sample": f"{rows} of {specs[0].M} token rows of each of the {len(specs)} GEMMs "
                      f"(all N, all K), {dt:.1f} s; rows are independent, so the whole workload "
                      f"would take about {dt * specs[0].M / rows:.0f} s",
            "seconds": dt}


def bench_chain(args):
    """Workload 5: the chained BERT-large linear stack at M = 32768.  A step is one encoder layer's four
    GEMMs (QKV, out-proj on the V third, FFN1+GELU, FFN2), each with the dequantize / bias (/GELU) /
    per-token requantize epilogue fused, codes flowing from one GEMM to the next without an fp16 tensor.
    Four layers with distinct weights are cycled; the step input is the previous layer's output."""
    import torch
    from paper_2301_12017_amd import binding as B, synth, workloads as WL
    B.lib()
    torch.cuda.set_device(0)
    M, h, ffn, nl = 32768, 1024, 4096, 4
    layout = B.preferred_layout(M, 3 * h, h)
    layers = WL.make_chain(nl, h, ffn, M, 5, keep_host=False, layout=layout)
    A0 = B.quantize_act(WL.dev(synth.activations(M, h, 0, 5, 0)), B.SYM, layout=layout)
    ws = torch.empty(M * 8, dtype=torch.uint8, device="cuda")
    # build the 16 calls once: run the chain eagerly and keep every output as the next call's input
    calls, names, A = [], [], A0
    for L in layers:
        for name, lay, slice_h in (("qkv", L.qkv, None), ("attn_out", L.out, h), ("ffn1", L.ffn1, None), ("ffn2", L.ffn2, None)):
            a_in = WL.v_slice(A, slice_h) if slice_h else A
            mfma = lay.W.layout == B.LAYOUT_MFMA
            out = B._alloc_out(a_in, lay.W, True, B.SYM, h if (mfma and name == "qkv") else 0, lay.W.layout)
            calls.append(B.PreparedLinear(a_in, lay.W, lay.bias, lay.act, requant=True, requant_mode=B.SYM,
                                          requant_group=h if (mfma and name == "qkv") else 0, out=out, workspace=ws,
                                          requant_layout=lay.W.layout))
            names.append(name)
            A = B.QAct(out[0], out[1], None, None, M, lay.spec.N, lay.spec.N // 2, 0, B.SYM, 0, lay.W.layout,
                       out[3] if mfma else None)
    stream = B._stream()
    steps = args.steps
    timers = [[B.KernelTimer() for _ in range(4)] for _ in range(steps)]

    def step(k, tm=None):
        for j in range(4):
            if tm:
                tm[j].arm()                                     # stamps the GEMM kernel's own start and end
            calls[(k % nl) * 4 + j](stream)

    settle(lambda: step(0), args.settle_ms)
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same steps once more with kernel-boundary events on every GEMM launch (roofline figure)
    for k in range(steps):
        step(k, timers[k])
    torch.cuda.synchronize()
    assert B.fused_fault_check() is False                       # no workgroup of a fused requantize gave up waiting
    ms = dt * 1e3 / steps
    shapes = [(3 * h, h), (h, h), (ffn, h), (h, ffn)]
    ops = sum(2 * M * n * k for n, k in shapes)
    gemm_ms = [sum(timers[k][j].elapsed_ms() for k in range(steps)) / steps for j in range(4)]
    achieved = ops / (sum(gemm_ms) * 1e-3) / 1e12
    line = {
        "metric": "W4A4 linear TOPS (% int8-MFMA peak); BERT-base layer latency b1/s128",
        "value": ops / (ms * 1e-3) / 1e12, "unit": "TOPS", "n_gpus": 1, "steps": steps, "warmup": args.warmup, "settle_ms": args.settle_ms,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 (int4 operands widened for the int8 MFMA, int32 accumulate, fp32 epilogue, int4 out)", "data": "synthetic",
        "config": {"workload": f"configs[4]: one layer of the chained BERT-large stack, M={M}: qkv, attn_out (V third in "
                               f"place), ffn1+GELU, ffn2, every output requantized per token in the GEMM epilogue",
                   "step": "4 x w4a4_linear(requant)", "layout": layout},
        "pct_int8_mfma_peak": 100.0 * ops / (ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS,
        "per_gemm": [{"name": n, "ms": t, "TOPS": 2 * M * nn * kk / (t * 1e-3) / 1e12}
                     for n, t, (nn, kk) in zip(names[:4], gemm_ms, shapes)],
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": achieved / INT8_MFMA_PEAK_TOPS, "traffic": None,
                     "kernel": "gemm_olay_kernel with the fused requantize epilogue, the four launches of the step",
                     "ops_per_step": ops, "kernel_ms_per_step": sum(gemm_ms)},
    }
    print(json.dumps(line))


def bench_curve(args):
    """Sec. 4.1 compares the INT4 with the INT8 GEMM over the token count M for the four encoder shapes.  Here: the
    fused linears (GEMM + dequantize + fp16 store, operands already quantized), kernel-boundary times."""
    import torch
    from paper_2301_12017_amd import binding as B, synth
    B.lib()
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda").manual_seed(0)
    reps = max(args.steps, 5)
    rows = []
    for model, h, ffn in (("bert-base", 768, 3072), ("bert-large", 1024, 4096)):
        for M in (128, 512, 1024, 2048, 4096, 8192, 12288, 16384):
            for spec in synth._encoder_linears(M, h, ffn):
                X = torch.randn((M, spec.K), device="cuda", generator=gen).half()
                W = (torch.randn((spec.N, spec.K), device="cuda", generator=gen) * 0.03).half()
                layout = B.preferred_layout(M, spec.N, spec.K)
                W4 = B.quantize_weight(W, B.SYM, 0, layout)
                A4 = B.quantize_act(X, B.SYM, layout=layout)
                c4 = B.PreparedLinear(A4, W4, schedule=args.schedule if layout == 1 else 0)
                w8 = B.quantize_rows8(W)
                a8 = B.quantize_rows8(X)
                c8 = B.PreparedLinear8(a8[0], a8[1], w8[0], w8[1])
                st = B._stream()
                us = {}
                for name, call in (("int4", c4), ("int8", c8)):
                    tms = [B.KernelTimer() for _ in range(reps)]
                    settle(lambda: call(st), min(args.settle_ms, 100.0))
                    for t in tms:
                        t.arm()
                        call(st)
                    torch.cuda.synchronize()
                    us[name] = sum(t.elapsed_ms() for t in tms) / reps * 1e3
                ops = 2.0 * M * spec.N * spec.K
                rows.append({"model": model, "M": M, "gemm": spec.name, "N": spec.N, "K": spec.K,
                             "int4_us": us["int4"], "int8_us": us["int8"],
                             "int4_TOPS": ops / us["int4"] / 1e6, "int8_TOPS": ops / us["int8"] / 1e6,
                             "int4_over_int8": us["int8"] / us["int4"]})
                del X, W, W4, A4, c4, w8, a8, c8
    print(json.dumps({"metric": "INT4 vs INT8 fused-linear kernel time over the token count (Sec. 4.1 shapes)", "unit": "us / TOPS",
                      "n_gpus": 1, "data": "synthetic", "reps": reps,
                      "note": "w4a4_linear against w8a8_linear on operands quantized beforehand, no bias, fp16 out; durations "
                              "from HIP events at the kernel's own start and end, mean of `reps` launches after up to 100 ms "
                              "of untimed launches of the same call",
                      "curve": rows}))


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the path is token-parallel with no "
              "exchange); --gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)
    if args.gemm_curve:
        return bench_curve(args)
    if args.config == 5:
        return bench_chain(args)
    import torch
    from paper_2301_12017_amd import binding as B, synth, workloads as WL
    B.lib()
    torch.cuda.set_device(0)
    cfg = args.config
    side_legs = cfg == 3 and not args.step_only
    specs = synth.config_linears(cfg)
    layers = [WL.make_layer(s, cfg, i, keep_host=False) for i, s in enumerate(specs)]
    Xs = [WL.dev(WL.make_input(s, cfg, i)) for i, s in enumerate(specs)]
    # everything the step touches is allocated once, outside the timed region
    qacts = [B.quantize_act(X, s.mode, s.group, layout=L.W.layout) for X, s, L in zip(Xs, specs, layers)]
    outs = [B._alloc_out(qa, L.W, False, 0, 0) for qa, L in zip(qacts, layers)]
    timers = [[B.KernelTimer() for _ in specs] for _ in range(args.steps)]

    # the calls of a step, with their arguments marshalled once (the timed loop only makes the C calls)
    stream = B._stream()
    q_calls = [B.PreparedQuantizeAct(X, qa) for X, qa in zip(Xs, qacts)]
    l_calls = [B.PreparedLinear(qa, L.W, L.bias, L.act, schedule=args.schedule, out=o)
               for qa, L, o in zip(qacts, layers, outs)]

    def step(tm=None, st=None):
        st = stream if st is None else st
        for i in range(len(specs)):
            q_calls[i](st)
            if tm:
                tm[i].arm()                                     # stamps the GEMM kernel's own start and end
            l_calls[i](st)

    settle(step, args.settle_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    ops = sum(2 * s.M * s.N * s.K for s in specs)
    tops = ops / (ms_per_step * 1e-3) / 1e12

    # the same steps once more with kernel-boundary HIP events on every w4a4_linear launch: the kernel
    # durations behind the roofline figure (what a kernel trace reports; no dispatch gap in them)
    for k in range(args.steps):
        step(timers[k])
    torch.cuda.synchronize()
    gemm_ms = [sum(timers[k][i].elapsed_ms() for k in range(args.steps)) / args.steps
               for i in range(len(specs))]
    gemm_tops = [2 * s.M * s.N * s.K / (t * 1e-3) / 1e12 for s, t in zip(specs, gemm_ms)]
    achieved = ops / (sum(gemm_ms) * 1e-3) / 1e12

    # ---- the same step replayed from a HIP graph (Sec. 4.2 names graph capture as the cure for launch
    # overhead): reported beside the eager figure, never instead of it
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(st=B._stream())
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            step(st=B._stream())
        settle(gr.replay, args.settle_ms)
        tg = time.perf_counter()
        for _ in range(args.steps):
            gr.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg) * 1e3 / args.steps
    except Exception as ex:                                       # report, never hide
        graph_ms = f"graph capture failed: {ex}"

    # ---- latency leg: BERT-base layer linears at batch 1 x seq 128 (launch/latency-bound)
    lat = {}
    if side_legs:
        s2 = synth.config_linears(2)
        l2 = [WL.make_layer(s, 2, i, keep_host=False) for i, s in enumerate(s2)]
        x2 = [WL.dev(WL.make_input(s, 2, i)) for i, s in enumerate(s2)]
        q2 = [B.quantize_act(X, s.mode, s.group) for X, s in zip(x2, s2)]
        o2 = [B._alloc_out(qa, L.W, False, 0, 0) for qa, L in zip(q2, l2)]

        qc2 = [B.PreparedQuantizeAct(X, qa) for X, qa in zip(x2, q2)]
        lc2 = [B.PreparedLinear(qa, L.W, L.bias, L.act, out=o) for qa, L, o in zip(q2, l2, o2)]

        def layer2():
            st = B._stream()
            for qc, lc in zip(qc2, lc2):
                qc(st)
                lc(st)
        lat_settle = min(args.settle_ms, 50.0)
        settle(layer2, lat_settle)
        reps = 200
        t1 = time.perf_counter()
        for _ in range(reps):
            layer2()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t1) * 1e6 / reps
        # the same eight launches replayed from a HIP graph (Sec. 4.2: a captured graph removes the
        # launch overhead that dominates at small batch x sequence)
        graph_us = None
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                layer2()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                layer2()
            for _ in range(5):
                gr.replay()
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for _ in range(reps):
                gr.replay()
            torch.cuda.synchronize()
            graph_us = (time.perf_counter() - t2) * 1e6 / reps
        except Exception as ex:                                   # report, never hide
            graph_us = f"graph capture failed: {ex}"
        # the same four linears through w4a4_linear_f16act: the activation quantize inside the GEMM kernel,
        # four launches instead of eight
        fc2 = [B.PreparedLinearF16Act(X, L.W, L.bias, L.act) for X, L in zip(x2, l2)]

        def layer2_fused():
            st = B._stream()
            for fc in fc2:
                fc(st)
        settle(layer2_fused, lat_settle)
        for fc, lc in zip(fc2, lc2):                                 # same bits as the two-call path
            assert torch.equal(fc.out.view(torch.int16), lc.out[0].view(torch.int16))
        t4 = time.perf_counter()
        for _ in range(reps):
            layer2_fused()
        torch.cuda.synchronize()
        fused_us = (time.perf_counter() - t4) * 1e6 / reps
        # floor of eight back-to-back launches on this stream: the smallest quantize_act the library accepts
        # (one token of 32 elements), eight times
        tiny_x = torch.zeros((1, 32), dtype=torch.float16, device="cuda")
        tiny = B.PreparedQuantizeAct(tiny_x, B.quantize_act(tiny_x, B.SYM))

        def eight():
            st = B._stream()
            for _ in range(8):
                tiny(st)
        settle(eight, lat_settle)
        t3 = time.perf_counter()
        for _ in range(reps):
            eight()
        torch.cuda.synchronize()
        floor_us = (time.perf_counter() - t3) * 1e6 / reps
        bytes2 = sum(s.M * s.K * 2 + s.M * s.K // 2 * 2 + s.N * s.K // 2 + s.M * s.N * 2 for s in s2)
        lat = {"bert_base_layer_b1_s128_us": fused_us, "bert_base_layer_b1_s128_two_call_us": us,
               "bert_base_layer_b1_s128_two_call_graph_us": graph_us,
               "eight_minimal_launches_us": floor_us,
               "algorithmic_bytes": bytes2,
               "achieved_GBps_warm": bytes2 / (fused_us * 1e-6) / 1e9,
               "note": "bert_base_layer_b1_s128_us: 4 x w4a4_linear_f16act (quantize_act inside the GEMM kernel, "
                       "one launch per linear, outputs identical to the two-call path); two_call: 4 x "
                       "(quantize_act + w4a4_linear), eager and replayed from a HIP graph; weights warm in cache; "
                       "attention, LayerNorm and residuals are outside the path; eight_minimal_launches_us = eight "
                       "one-token quantize_act launches, the launch floor of eight launches on this stream"}

    # ---- whole encoder layer at batch 1 x seq 128 (Sec. 4.2: FP16 attention and LayerNorms around the four linears,
    # the launch sequence replayed from a graph): w4a4_encoder_layer, eager and from a HIP graph, under the strategy
    # the library's table names for this shape and, for comparison, with every part in the INT8 sibling
    whole = {}
    if side_legs:
        bsz, sq, hd, hh, ff = 1, 128, 12, 768, 3072
        gen = torch.Generator(device="cuda").manual_seed(1)
        rn = lambda *shape, std=1.0: (torch.randn(shape, device="cuda", generator=gen) * std).half()
        enc = B.EncoderLayer(bsz, sq, hd, rn(3 * hh, hh, std=0.03), rn(3 * hh, std=0.02), rn(hh, hh, std=0.03), rn(hh, std=0.02),
                             rn(ff, hh, std=0.03), rn(ff, std=0.02), rn(hh, ff, std=0.03), rn(hh, std=0.02),
                             (1 + 0.1 * torch.randn(hh, device="cuda", generator=gen)).half(), rn(hh, std=0.1),
                             (1 + 0.1 * torch.randn(hh, device="cuda", generator=gen)).half(), rn(hh, std=0.1))
        xin = rn(bsz * sq, hh)
        yout = torch.empty_like(xin)
        pick = B.strategy_lookup(bsz * sq, hh, ff)
        reps = 200
        for name, strat_ in (("int4", pick), ("int8", 0)):
            settle(lambda: enc(xin, strat_, out=yout), lat_settle)
            eager = yout.clone()
            tw = time.perf_counter()
            for _ in range(reps):
                enc(xin, strat_, out=yout)
            torch.cuda.synchronize()
            whole[f"{name}_eager_us"] = (time.perf_counter() - tw) * 1e6 / reps
            try:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    enc(xin, strat_, out=yout, stream=side.cuda_stream)
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                gw = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gw, stream=side):
                    enc(xin, strat_, out=yout, stream=side.cuda_stream)
                for _ in range(5):
                    gw.replay()
                torch.cuda.synchronize()
                assert torch.equal(yout, eager)                      # a replay gives the eager result
                tw = time.perf_counter()
                for _ in range(reps):
                    gw.replay()
                torch.cuda.synchronize()
                whole[f"{name}_graph_us"] = (time.perf_counter() - tw) * 1e6 / reps
            except Exception as ex:                                   # report, never hide
                whole[f"{name}_graph_us"] = f"graph capture failed: {ex}"
        whole["strategy"] = pick
        whole["note"] = ("one post-LN BERT-base encoder layer, batch 1 x seq 128, fp16 in / fp16 out: qkv, FP16 attention "
                         "stand-in (no mask), attention output, residual + LayerNorm, ffn1 + GELU, ffn2, residual + LayerNorm "
                         "= 7 launches in either precision (quantize inside the GEMM kernels); back-to-back calls, weights warm")

    # ---- producer fusion (Sec. 4.2): LayerNorm(x + residual) fused with the token-wise quantize, at the
    # hidden size of this workload; HBM-bound, so it is reported against the HBM peak.  Four rotating
    # buffer sets (> the 256 MB on-package cache) so that nothing is served from cache.
    ln = {}
    if side_legs:
        Mh, Kh, nset = specs[0].M, specs[0].K, 4
        rng_t = torch.Generator(device="cuda").manual_seed(0)
        sets = []
        for _ in range(nset):
            x = torch.randn((Mh, Kh), device="cuda", generator=rng_t).half()
            r = torch.randn((Mh, Kh), device="cuda", generator=rng_t).half()
            g = (1.0 + 0.1 * torch.randn((Kh,), device="cuda", generator=rng_t)).half()
            b = (0.1 * torch.randn((Kh,), device="cuda", generator=rng_t)).half()
            out = B._new_qact(Mh, Kh, B.SYM, 0, layers[0].W.layout, x.device)
            y = torch.empty((Mh, Kh), dtype=torch.float16, device="cuda")
            sets.append(B.PreparedLayerNormQuantize(x, r, g, b, 1e-12, out, y))
        settle(lambda: [c(stream) for c in sets], lat_settle)
        reps_ln = 200
        t5 = time.perf_counter()
        for i in range(reps_ln):
            sets[i % nset](stream)
        torch.cuda.synchronize()
        ln_us = (time.perf_counter() - t5) * 1e6 / reps_ln
        ln_bytes = Mh * Kh * (2 + 2 + 2) + Mh * Kh // 2 + Mh * 8 + 2 * Kh * 2
        ln = {"layernorm_quantize_us": ln_us, "shape": [Mh, Kh], "algorithmic_bytes": ln_bytes,
              "achieved_GBps": ln_bytes / (ln_us * 1e-6) / 1e9, "frac_of_hbm_peak": ln_bytes / (ln_us * 1e-6) / 8e12,
              "note": "w4a4_layernorm_quantize with residual and fp16 copy; back-to-back launches over four "
                      "rotating buffer sets, launch gaps included"}

    # ---- the INT8 sibling on the same workload (the paper's Sec. 4.1 comparison, on this hardware): the same
    # step with w8a8_quantize_rows + w8a8_linear, timed the same way
    i8 = {}
    if side_legs:
        w8 = [B.quantize_rows8(WL.dev(WL.make_layer(s_, cfg, i, keep_host=True).host_W)) for i, s_ in enumerate(specs)]
        a8 = [B.quantize_rows8(X) for X in Xs]
        q8_calls = [B.PreparedQuantizeRows8(X, a[0], a[1]) for X, a in zip(Xs, a8)]
        l8_calls = [B.PreparedLinear8(a[0], a[1], w[0], w[1], L.bias, L.act, out=o[0])
                    for a, w, L, o in zip(a8, w8, layers, outs)]
        t8 = [[B.KernelTimer() for _ in specs] for _ in range(args.steps)]

        def step8(tm=None):
            for i in range(len(specs)):
                q8_calls[i](stream)
                if tm:
                    tm[i].arm()
                l8_calls[i](stream)
        settle(step8, args.settle_ms)
        for _ in range(args.warmup):
            step8()
        torch.cuda.synchronize()
        t6 = time.perf_counter()
        for _ in range(args.steps):
            step8()
        torch.cuda.synchronize()
        ms8 = (time.perf_counter() - t6) * 1e3 / args.steps
        for k in range(args.steps):
            step8(t8[k])
        torch.cuda.synchronize()
        g8 = [sum(t8[k][i].elapsed_ms() for k in range(args.steps)) / args.steps for i in range(len(specs))]
        i8 = {"ms_per_step": ms8, "TOPS": ops / (ms8 * 1e-3) / 1e12, "kernel_ms_per_step": sum(g8),
              "frac_of_int8_mfma_peak": ops / (sum(g8) * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS,
              "per_gemm_ms": {s_.name: t for s_, t in zip(specs, g8)},
              "int4_over_int8_gemm_speedup": sum(g8) / sum(gemm_ms),
              "note": "w8a8_quantize_rows + w8a8_linear on the same inputs and shapes; both paths use the int8 "
                      "MFMA, INT4 halves the operand bytes and pays for the nibble widening"}

    # ---- context only: the vendor library's FP16 GEMM (torch.matmul -> hipBLASLt) on the same four shapes, the
    # precision the paper's speedups are quoted against.  Plain matmul: no bias, no GELU, no quantize.
    fp16 = {}
    if side_legs:
        try:
            Wh = [torch.randn((s_.N, s_.K), device="cuda").half() * 0.02 for s_ in specs]
            Yh = [torch.empty((s_.M, s_.N), dtype=torch.float16, device="cuda") for s_ in specs]
            settle(lambda: [torch.matmul(X, W_.t(), out=Y_) for X, W_, Y_ in zip(Xs, Wh, Yh)], args.settle_ms)   # same treatment
            t7 = time.perf_counter()
            for _ in range(args.steps):
                for X, W_, Y_ in zip(Xs, Wh, Yh):
                    torch.matmul(X, W_.t(), out=Y_)
            torch.cuda.synchronize()
            ms16 = (time.perf_counter() - t7) * 1e3 / args.steps
            fp16 = {"ms_per_step": ms16, "TFLOPS": ops / (ms16 * 1e-3) / 1e12,
                    "w4a4_step_speedup": ms16 / ms_per_step,
                    "note": "four torch.matmul calls (hipBLASLt FP16, fp32 accumulate) on the same activations and "
                            "shapes, launch gaps included; the W4A4 step it is compared with also contains the four "
                            "quantize_act kernels, bias and GELU"}
        except Exception as ex:                                   # context only: never fail the bench over it
            fp16 = {"error": str(ex)}
        try:                                                          # and its INT8 GEMM (int32 out, no epilogue)
            a8l = [a[0] for a in a8]
            w8l = [w[0].t() for w in w8]
            settle(lambda: [torch._int_mm(a_, w_) for a_, w_ in zip(a8l, w8l)], args.settle_ms)
            t8l = time.perf_counter()
            for _ in range(args.steps):
                for a_, w_ in zip(a8l, w8l):
                    torch._int_mm(a_, w_)
            torch.cuda.synchronize()
            ms8l = (time.perf_counter() - t8l) * 1e3 / args.steps
            fp16["int8_library_gemm_ms_per_step"] = ms8l
            fp16["int8_library_gemm_TOPS"] = ops / (ms8l * 1e-3) / 1e12
        except Exception as ex:
            fp16["int8_library_gemm_error"] = str(ex)[:200]

    # ---- per-part strategy (Sec. 4.2 / 4.3): every part timed in INT4 and in the INT8 sibling, the FFN pair also with
    # the codes handed over in the epilogue, at the paper's annotated (batch-sequence) points for BERT-base and at
    # this bench's own token count; the library's tuner does the timing and the picking
    strat = {}
    if side_legs:
        names = ["qkv", "attn_out", "ffn1", "ffn2"]
        points = [("1-32", 32, 768, 3072), ("1-128", 128, 768, 3072), ("8-32", 256, 768, 3072),
                  ("16-128", 2048, 768, 3072), ("128-128", 16384, 768, 3072),
                  ("bench", specs[0].M, specs[0].K, specs[2].N)]
        rows = []
        for tag, M_, h_, f_ in points:
            pick, part_us, fused_us = B.strategy_tune(M_, h_, f_, iters=20)
            rows.append({"bs_seq": tag, "M": M_, "hidden": h_, "ffn": f_,
                         "int8_us": {n: part_us[i][0] for i, n in enumerate(names)},
                         "int4_us": {n: part_us[i][1] for i, n in enumerate(names)},
                         "ffn_fused_int4_us": fused_us, "strategy": pick,
                         "int4_parts": [n for i, n in enumerate(names) if pick >> i & 1],
                         "ffn_fused": bool(pick & B.STRATEGY_FUSED_FFN)})
        strat = {"points": rows,
                 "note": "w4a4_strategy_tune: each option = quantize + linear from fp16 to fp16 on synthetic operands, "
                         "20 timed runs back to back; the paper's GPU wanted only ffn1 in INT4 at the three smallest points"}

    line = {
        "metric": "W4A4 linear TOPS (% int8-MFMA peak); BERT-base layer latency b1/s128",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_ms": args.settle_ms,
        "ms_per_step": ms_per_step, "ms_per_step_graph_replay": graph_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 (int4 operands widened for the int8 MFMA, int32 accumulate, fp32 epilogue, fp16 out)",
        "data": "synthetic",
        "config": {"workload": f"configs[{cfg - 1}]: " + ", ".join(f"{s.name} {s.M}x{s.N}x{s.K}" for s in specs)
                   + ("; symmetric per-token / per-channel INT4" if cfg != 4 else
                      "; asymmetric INT4, weight groups of 128, 8 outlier channels x20"),
                   "step": "quantize_act + w4a4_linear (fused GEMM, dequant, bias, GELU on ffn1, fp16 store) x 4",
                   "schedule": args.schedule},
        "pct_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
        "per_gemm": [{"name": s.name, "ms": t, "TOPS": g} for s, t, g in zip(specs, gemm_ms, gemm_tops)],
        "latency": lat,
        "whole_layer_b1_s128": whole,
        "producer_fusion": ln,
        "int8_sibling": i8,
        "per_part_strategy": strat,
        "fp16_library_gemm": fp16,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": achieved / INT8_MFMA_PEAK_TOPS,
                     "traffic": PROFILED_TRAFFIC_BYTES.get(cfg) if args.schedule == 0 else None,
                     "traffic_unit": "bytes per step (the four launches), profiled separately",
                     "kernel": "gemm_olay_kernel (w4a4_linear), the four launches of the step"
                               if cfg in (3, 5) else "gemm_kernel (w4a4_linear), the four launches of the step",
                     "ops_per_step": ops, "kernel_ms_per_step": sum(gemm_ms)},
    }
    if args.copy_probe_mb:
        src = torch.empty(args.copy_probe_mb << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(specs, cfg, args.cpu_rows)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
