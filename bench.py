#!/usr/bin/env python3
"""Benchmark of the W4A4 linear hot path on one MI355X.

A step is one pass of the whole path -- token-wise quantize_act, then the fused
INT4 GEMM + dequantize/bias(/GELU) epilogue with an fp16 store -- over the four
encoder linears of BERT-large at batch 32 x seq 384 (M = 12288; Sec. 4.1 shapes),
with fp16 activations, quantized weights and biases already resident in HBM.
`value` is 2*M*N*K summed over the four GEMMs divided by the step time (so the
quantize kernels count against it).  The line also carries
  roofline         the GEMM kernels of the step against the int8 MFMA peak (HIP events at each kernel's own
                   start and end), beside the ceilings measured in the same run (`ceilings`);
  latency          the BERT-base layer linears at batch 1 x seq 128, warm and cold;
  other_workloads  short legs of the asymmetric / grouped workload and of the chained requantizing stack;
  cpu_baseline     the CPU oracle timed on a sample of token rows of the same workload, on all host cores
                   and on one.
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
FP6_MFMA_PEAK_TOPS = 10100.0      # MI355X dense FP6 / FP4 matrix peak, 10.1 PFLOP/s
HBM_PEAK_GBS = 8000.0
METRIC = "W4A4 linear TOPS (% int8-MFMA peak); BERT-base layer latency b1/s128"
DTYPE = "int8 (int4 operands widened for the int8 MFMA, int32 accumulate, fp32 epilogue, {} out)"
DTYPE_FP6 = "fp6 (int4 codes as FP6 E2M3 operands of the f8f6f4 MFMA, fp32 accumulate: exact integer sums, fp32 epilogue, {} out)"
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemm_config3_hbm_traffic.txt")


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=300)
    p.add_argument("--warmup", type=int, default=10)
    p.add_argument("--config", type=int, default=3, help="workload number (3 = headline, 4 = asymmetric/grouped, 5 = one layer of the chained stack)")
    p.add_argument("--schedule", type=int, default=0, help="force a GEMM tile schedule (0 = built-in table)")
    p.add_argument("--layout", type=int, default=-1,
                   help="operand layout of the step's layers (-1 = what the library prefers for the shape; 0 canonical, "
                        "1 int8-MFMA operand layout, 2 FP6 operand layout)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--settle-ms", type=float, default=300.0,
                   help="untimed steps run for this long before the warm-up steps: after an idle phase the chip's "
                        "clocks dip for some milliseconds a few milliseconds into a burst of work, and a short timed "
                        "region that starts right after set-up would measure that transient instead of the sustained rate")
    p.add_argument("--gemm-curve", action="store_true",
                   help="instead of the step: INT4 and INT8 GEMM kernel time over the token count for the BERT-base and "
                        "BERT-large shapes (the comparison of Sec. 4.1 on this hardware); prints its own JSON line")
    p.add_argument("--step-only", action="store_true",
                   help="only the timed step and its roofline: skip every side leg (for profiler runs, so that a kernel "
                        "trace holds the step's launches alone)")
    p.add_argument("--latency-only", action="store_true",
                   help="only the batch 1 x seq 128 latency leg (for profiler runs of the M = 128 kernels); prints its own JSON line")
    p.add_argument("--quantize-only", action="store_true",
                   help="only the token-wise quantizer at the workload's shapes, over rotating inputs (for profiler runs); "
                        "prints its own JSON line")
    p.add_argument("--copy-probe-mb", type=int, default=0,
                   help="also run one plain device copy of this many MiB (a kernel of known traffic, used to "
                        "calibrate the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    p.add_argument("--cpu-rows", type=int, default=256, help="token rows per GEMM and worker the oracle is timed on")
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


# ------------------------------------------------------------------------------------------ CPU oracle
def _oracle_rows(job):
    """One worker: the oracle's quantize_act + linear on `rows` token rows of every GEMM of the workload.
    Returns the seconds the timed part took (weights are quantized beforehand, an offline step)."""
    cfg, rows, worker = job
    import oracle
    from paper_2301_12017_amd import synth
    specs = synth.config_linears(cfg)
    prepared = []
    for i, s in enumerate(specs):
        X = synth.activations(rows, s.K, worker, cfg, 10 * i, outlier_channels=8 if cfg == 4 else 0)
        W = synth.weights(s.N, s.K, 0, cfg, 10 * i + 1)
        b = synth.bias(s.N, 0, cfg, 10 * i + 2)
        prepared.append((s, X, oracle.quantize_weight(W, s.mode, s.group), b))
    t0 = time.perf_counter()
    for s, X, Q, b in prepared:
        A = oracle.quantize_act(X, s.mode, s.group)
        oracle.linear(A, Q, s.mode, s.group, b, oracle.ACT_GELU if s.gelu else oracle.ACT_NONE)
    return time.perf_counter() - t0


def host_cores():
    """Worker count for the all-core figure: the machine's CPU share (the scheduler affinity of this process, capped by
    OMP_NUM_THREADS where the environment sets it)."""
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    try:
        cap = int(os.environ.get("OMP_NUM_THREADS", "0"))
    except ValueError:
        cap = 0
    return max(1, min(n, cap) if cap > 0 else n)


def cpu_baseline(cfg, rows):
    """The oracle as it stands (plain C, one thread per process) on a sample of token rows of every GEMM: once on a
    single core, once on all cores (one worker process per core, each with its own `rows` rows; token rows are
    independent end to end).  Must run before this process touches the GPU: the workers are forked."""
    import multiprocessing as mp
    from paper_2301_12017_amd import synth
    import oracle
    specs = synth.config_linears(cfg)
    ops_per_row = sum(2 * s.N * s.K for s in specs)
    oracle.lib()                                                      # compiled before the workers start
    one = _oracle_rows((cfg, rows, 0))
    cores = host_cores()
    t0 = time.perf_counter()
    with mp.get_context("fork").Pool(cores) as pool:
        secs = pool.map(_oracle_rows, [(cfg, rows, w) for w in range(cores)], chunksize=1)
    wall = time.perf_counter() - t0
    span = max(secs)                                                  # the timed part of the slowest worker
    return {"value": ops_per_row * rows * cores / span / 1e12, "unit": "TOPS", "cores": cores, "kind": "oracle",
            "sample": f"{rows} token rows of each of the {len(specs)} GEMMs (all N, all K) per worker process, {cores} "
                      f"workers = {rows * cores} of {specs[0].M} rows, {span:.1f} s (slowest worker; {wall:.1f} s with "
                      f"set-up); rows are independent, so the whole workload would take about "
                      f"{span * specs[0].M / (rows * cores):.0f} s on these cores",
            "seconds": span,
            "single_thread": {"value": ops_per_row * rows / one / 1e12, "unit": "TOPS", "cores": 1, "seconds": one,
                              "sample": f"{rows} token rows of each GEMM"},
            "host_cores_visible": os.cpu_count()}


# ------------------------------------------------------------------------------------------ workloads 3 and 4
KERNEL_NAMES = {"olay": "gemm_olay_kernel", "group": "gemm_group_kernel", "pipe": "gemm_pipe_kernel",
                "generic": "gemm_kernel", "small": "linear_f16act_kernel", "fp6": "gemm_fp6_kernel"}


def kernel_label(schedules):
    fam = sorted({n.split("_")[0] for n in schedules})
    return " / ".join(KERNEL_NAMES.get(f, f) for f in fam) + " (w4a4_linear), the four launches of the step; schedules " \
        + ", ".join(schedules)


class StepWorkload:
    """quantize_act + w4a4_linear for the four linears of workload `cfg`, everything allocated and marshalled once."""

    def __init__(self, cfg, schedule=0, layout=-1):
        import torch
        from paper_2301_12017_amd import binding as B, synth, workloads as WL
        self.cfg, self.B = cfg, B
        self.specs = synth.config_linears(cfg)
        # layout: -1 = what the library prefers per shape, a number = that layout for every layer, a list = per layer
        lays = layout if isinstance(layout, (list, tuple)) else [layout] * len(self.specs)
        self.layers = [WL.make_layer(s, cfg, i, keep_host=False, layout=None if lay < 0 else lay)
                       for i, (s, lay) in enumerate(zip(self.specs, lays))]
        self.Xs = [WL.dev(WL.make_input(s, cfg, i)) for i, s in enumerate(self.specs)]
        self.qacts = [B.quantize_act(X, s.mode, s.group, layout=L.W.layout) for X, s, L in zip(self.Xs, self.specs, self.layers)]
        self.outs = [B._alloc_out(qa, L.W, False, 0, 0) for qa, L in zip(self.qacts, self.layers)]
        self.q_calls = [B.PreparedQuantizeAct(X, qa) for X, qa in zip(self.Xs, self.qacts)]
        self.l_calls = [B.PreparedLinear(qa, L.W, L.bias, L.act, schedule=schedule, out=o)
                        for qa, L, o in zip(self.qacts, self.layers, self.outs)]
        self.schedules = [B.pick_schedule(qa, L.W, schedule=schedule) for qa, L in zip(self.qacts, self.layers)]
        self.stream = B._stream()
        self.ops = sum(2 * s.M * s.N * s.K for s in self.specs)
        torch.cuda.synchronize()

    def step(self, tm=None, st=None):
        st = self.stream if st is None else st
        for i in range(len(self.specs)):
            self.q_calls[i](st)
            if tm:
                tm[i].arm()                                     # stamps the GEMM kernel's own start and end
            self.l_calls[i](st)

    def measure(self, steps, warmup, settle_ms):
        import torch
        B = self.B
        settle(self.step, settle_ms)
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # the same steps once more with kernel-boundary HIP events on every w4a4_linear launch: the kernel
        # durations behind the roofline figure (what a kernel trace reports; no dispatch gap in them)
        timers = [[B.KernelTimer() for _ in self.specs] for _ in range(steps)]
        for k in range(steps):
            self.step(timers[k])
        torch.cuda.synchronize()
        gemm_ms = [sum(timers[k][i].elapsed_ms() for k in range(steps)) / steps for i in range(len(self.specs))]
        ms = dt * 1e3 / steps
        return {"ms_per_step": ms, "timed_region_s": dt, "TOPS": self.ops / (ms * 1e-3) / 1e12, "gemm_ms": gemm_ms,
                "kernel_ms_per_step": sum(gemm_ms), "achieved_TOPS": self.ops / (sum(gemm_ms) * 1e-3) / 1e12}


def profiled_traffic(schedules):
    """HBM-side bytes of the four w4a4_linear launches of one step of the headline workload, from the rocprofv3 --pmc
    summary under profiles/ -- only if that summary was taken on the schedules this run uses (its `schedules:` line),
    else None: the figure is not measured live."""
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None
    got_s = got_b = None
    for line in text.splitlines():
        if line.startswith("schedules:"):
            got_s = [t.strip() for t in line.split(":", 1)[1].split(",")]
        if line.startswith("traffic_bytes_per_step:"):
            got_b = int(line.split(":", 1)[1].split()[0])
    return got_b if got_s == list(schedules) else None


# ------------------------------------------------------------------------------------------ workload 5
def chain_leg(steps, warmup, settle_ms, layout=None):
    """Workload 5: the chained BERT-large linear stack at M = 32768.  A step is one encoder layer's four
    GEMMs (QKV, out-proj on the V third, FFN1+GELU, FFN2), each with the dequantize / bias (/GELU) /
    per-token requantize epilogue fused, codes flowing from one GEMM to the next without an fp16 tensor.
    Four layers with distinct weights are cycled; the step input is the previous layer's output.
    `layout`: the operand layout of every GEMM and of every requantized output (default: the one the library prefers
    on the int8 MFMA; the FP6 layout runs the chain on the FP6 matrix instruction)."""
    import torch
    from paper_2301_12017_amd import binding as B, synth, workloads as WL
    M, h, ffn, nl = 32768, 1024, 4096, 4
    if layout is None or layout < 0:
        layout = B.preferred_layout(M, 3 * h, h)
    layers = WL.make_chain(nl, h, ffn, M, 5, keep_host=False, layout=layout)
    A0 = B.quantize_act(WL.dev(synth.activations(M, h, 0, 5, 0)), B.SYM, layout=layout)
    ws = torch.empty(M * 8, dtype=torch.uint8, device="cuda")
    # build the 16 calls once: run the chain eagerly and keep every output as the next call's input
    calls, names, A, scheds = [], [], A0, []
    for L in layers:
        for name, lay, slice_h in (("qkv", L.qkv, None), ("attn_out", L.out, h), ("ffn1", L.ffn1, None), ("ffn2", L.ffn2, None)):
            a_in = WL.v_slice(A, slice_h) if slice_h else A
            mfma = lay.W.layout == B.LAYOUT_MFMA
            rg = h if (mfma and name == "qkv") else 0
            out = B._alloc_out(a_in, lay.W, True, B.SYM, rg, lay.W.layout)
            calls.append(B.PreparedLinear(a_in, lay.W, lay.bias, lay.act, requant=True, requant_mode=B.SYM,
                                          requant_group=rg, out=out, workspace=ws, requant_layout=lay.W.layout))
            scheds.append(B.pick_schedule(a_in, lay.W, requant=True, requant_group=rg, requant_layout=lay.W.layout))
            names.append(name)
            A = B.QAct(out[0], out[1], None, None, M, lay.spec.N, B._row_bytes(lay.spec.N, lay.W.layout), 0, B.SYM, 0, lay.W.layout,
                       out[3] if mfma else None)
    stream = B._stream()

    def step(k, tm=None):
        for j in range(4):
            if tm:
                tm[j].arm()                                     # stamps the GEMM kernel's own start and end
            calls[(k % nl) * 4 + j](stream)

    settle(lambda: step(0), settle_ms)
    for k in range(warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(k)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    timers = [[B.KernelTimer() for _ in range(4)] for _ in range(steps)]
    for k in range(steps):
        step(k, timers[k])
    torch.cuda.synchronize()
    assert B.fused_fault_check() is False                       # no workgroup of a fused requantize gave up waiting
    ms = dt * 1e3 / steps
    shapes = [(3 * h, h), (h, h), (ffn, h), (h, ffn)]
    ops = sum(2 * M * n * k for n, k in shapes)
    gemm_ms = [sum(timers[k][j].elapsed_ms() for k in range(steps)) / steps for j in range(4)]
    return {"M": M, "layout": layout, "ms_per_step": ms, "timed_region_s": dt, "ops": ops, "TOPS": ops / (ms * 1e-3) / 1e12,
            "gemm_ms": gemm_ms, "names": names[:4], "shapes": shapes, "schedules": scheds[:4],
            "kernel_ms_per_step": sum(gemm_ms), "achieved_TOPS": ops / (sum(gemm_ms) * 1e-3) / 1e12}


def bench_chain(args):
    import torch
    from paper_2301_12017_amd import binding as B
    B.lib()
    torch.cuda.set_device(0)
    r = chain_leg(args.steps, args.warmup, args.settle_ms, args.layout)
    M = r["M"]
    fp6 = r["layout"] == B.LAYOUT_FP6
    line = {
        "metric": METRIC, "value": r["TOPS"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_ms": args.settle_ms, "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": (DTYPE_FP6 if fp6 else DTYPE).format("int4"), "data": "synthetic",
        "config": {"workload": f"configs[4]: one layer of the chained BERT-large stack, M={M}: qkv, attn_out (V third in "
                               f"place), ffn1+GELU, ffn2, every output requantized per token in the GEMM epilogue",
                   "step": "4 x w4a4_linear(requant)", "layout": r["layout"]},
        "pct_int8_mfma_peak": 100.0 * r["TOPS"] / INT8_MFMA_PEAK_TOPS,
        "per_gemm": [{"name": n, "ms": t, "TOPS": 2 * M * nn * kk / (t * 1e-3) / 1e12,
                      "frac": 2 * M * nn * kk / (t * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS}
                     for n, t, (nn, kk) in zip(r["names"], r["gemm_ms"], r["shapes"])],
        "roofline": {"bound": "mfma", "achieved": r["achieved_TOPS"], "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": r["achieved_TOPS"] / INT8_MFMA_PEAK_TOPS, "traffic": None,
                     "kernel": ("gemm_fp6_kernel" if fp6 else "gemm_olay_kernel")
                               + " with the fused requantize epilogue, the four launches of the step; schedules "
                               + ", ".join(r["schedules"]),
                     "ops_per_step": r["ops"], "kernel_ms_per_step": r["kernel_ms_per_step"]},
        "consistency": {"timed_region_s": r["timed_region_s"]},
    }
    print(json.dumps(line))


# ------------------------------------------------------------------------------------------ measured ceilings
def ceilings_leg(settle_ms):
    """What the device delivers on its own, in this run: the matrix pipe in a register-only MFMA loop (all-zero
    operands, and INT4 codes with the value distribution of quantized Gaussian data, widened as the GEMM kernels widen
    them), and the memory system under a coalesced read-only stream and a copy."""
    import numpy as np
    import torch
    from paper_2301_12017_amd import binding as B
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(0)
    codes = np.clip(np.rint(rng.standard_normal((64, 16, 4)) * 1.9), -7, 7).astype(np.int64)   # per lane, per word, per byte
    lo = (codes + 8) & 0xF                                            # offset-binary low nibbles: code + 8
    hi = (codes & 0xF) << 4                                           # two's-complement high nibbles: 16 * code as int8
    pick = np.zeros((64, 16), dtype=bool)                             # A operands: low type in even words; B: in odd words
    for w in range(16):
        pick[:, w] = ((w % 2) == 0) != ((w % 8) >= 4)
    bytes_ = np.where(pick[:, :, None], lo, hi).astype(np.uint32)
    words = (bytes_[:, :, 0] | (bytes_[:, :, 1] << 8) | (bytes_[:, :, 2] << 16) | (bytes_[:, :, 3] << 24)).astype(np.uint32)
    ops_real = torch.from_numpy(words.view(np.int32).copy()).cuda()
    ops_zero = torch.zeros_like(ops_real)
    out = {}
    iters = 4000
    # the same codes as FP6 E2M3 fields (sign, then the magnitude's exponent and mantissa), 32 per operand
    mag6 = np.array([0, 8, 16, 20, 24, 26, 28, 30], dtype=np.uint8)
    c6 = np.clip(np.rint(rng.standard_normal((64, 4, 32)) * 1.9), -7, 7).astype(np.int64)      # per lane: A0, B0, A1, B1
    f6 = (np.where(c6 < 0, 32, 0) | mag6[np.abs(c6)]).astype(np.uint8)
    bits6 = ((f6[..., None] >> np.arange(6, dtype=np.uint8)) & 1).astype(np.uint8).reshape(64, 4, 192)
    bytes6 = np.packbits(bits6, axis=2, bitorder="little")                                      # [64, 4, 24]
    ops6 = np.zeros((64, 4, 32), dtype=np.uint8)
    ops6[:, :, :24] = bytes6
    ops6_real = torch.from_numpy(ops6.reshape(64, 128).view(np.int32).copy()).cuda()            # [64 lanes][32 words]
    for name, ops in (("zero_operands", torch.zeros_like(ops6_real)), ("int4_codes", ops6_real)):
        settle(lambda: B.probe_mfma_fp6(ops, 500, sink), min(settle_ms, 100.0))
        tms = [B.KernelTimer() for _ in range(5)]
        n = 0
        for t in tms:
            t.arm()
            n = B.probe_mfma_fp6(ops, iters, sink)
        torch.cuda.synchronize()
        ms = sorted(t.elapsed_ms() for t in tms)[len(tms) // 2]
        out[f"mfma_fp6_{name}_TOPS"] = n * 131072.0 / (ms * 1e-3) / 1e12
    for name, ops in (("zero_operands", ops_zero), ("int4_codes", ops_real)):
        settle(lambda: B.probe_mfma(ops, 500, sink), min(settle_ms, 100.0))
        tms = [B.KernelTimer() for _ in range(5)]
        n = 0
        for t in tms:
            t.arm()
            n = B.probe_mfma(ops, iters, sink)
        torch.cuda.synchronize()
        ms = sorted(t.elapsed_ms() for t in tms)[len(tms) // 2]
        out[f"mfma_{name}_TOPS"] = n * 65536.0 / (ms * 1e-3) / 1e12
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty(nbytes // 2, dtype=torch.uint8, device="cuda")
    for name, s_, d_, moved in (("read", src, None, nbytes), ("copy", src[:nbytes // 2], dst, nbytes)):
        settle(lambda: B.probe_stream(s_, d_, sink), min(settle_ms, 50.0))
        tms = [B.KernelTimer() for _ in range(5)]
        for t in tms:
            t.arm()
            B.probe_stream(s_, d_, sink)
        torch.cuda.synchronize()
        ms = sorted(t.elapsed_ms() for t in tms)[len(tms) // 2]
        out[f"hbm_{name}_GBps"] = moved / (ms * 1e-3) / 1e9
    out["note"] = ("register-only v_mfma_i32_32x32x32_i8 loop, two waves per SIMD on every CU (w4a4_probe_mfma), and the same loop of "
                   "v_mfma_f32_32x32x64_f8f6f4 on FP6 E2M3 operands (w4a4_probe_mfma_fp6; nominal 10100 TOP/s), median of five "
                   "launches; a coalesced 1 GiB read-only stream and a 512 MiB -> 512 MiB copy (w4a4_probe_stream, bytes "
                   "read + written); nominal peaks: 5000 TOP/s, 8000 GB/s")
    del src, dst
    return out


# ------------------------------------------------------------------------------------------ latency (workload 2)
def latency_leg(settle_ms, cold_sets=96):
    """BERT-base layer linears at batch 1 x seq 128 (configs[1]): launch- and latency-bound."""
    import torch
    from paper_2301_12017_amd import binding as B, synth, workloads as WL
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
    lat_settle = min(settle_ms, 50.0)
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
    # kernel-boundary durations of the four one-launch linears (what a kernel trace reports)
    ktm = [[B.KernelTimer() for _ in fc2] for _ in range(20)]
    for row in ktm:
        st = B._stream()
        for t, fc in zip(row, fc2):
            t.arm()
            fc(st)
    torch.cuda.synchronize()
    kernel_us = [sum(row[i].elapsed_ms() for row in ktm) / len(ktm) * 1e3 for i in range(len(fc2))]
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
    # cold: `cold_sets` distinct sets of activations, weights, biases and outputs (about 6.7 MB each, 640 MB in all:
    # more than the L2 caches and the on-package cache hold), visited round robin, so that every launch fetches its
    # operands from HBM
    gen = torch.Generator(device="cuda").manual_seed(2)
    sets = []
    for _ in range(cold_sets):
        calls = []
        for s, L in zip(s2, l2):
            X = torch.randn((s.M, s.K), device="cuda", generator=gen).half()
            W = B.quantize_weight((torch.randn((s.N, s.K), device="cuda", generator=gen) * 0.02).half(), B.SYM)
            b = (torch.randn((s.N,), device="cuda", generator=gen) * 0.01).half()
            calls.append(B.PreparedLinearF16Act(X, W, b, L.act))
        sets.append(calls)
    torch.cuda.synchronize()

    def cold_pass():
        st = B._stream()
        for calls in sets:
            for c in calls:
                c(st)
    cold_pass()
    torch.cuda.synchronize()
    t5 = time.perf_counter()
    for _ in range(2):
        cold_pass()
    torch.cuda.synchronize()
    cold_us = (time.perf_counter() - t5) * 1e6 / (2 * cold_sets)
    bytes1 = [s.M * s.K * 2 + s.N * s.K // 2 + s.M * s.N * 2 + s.N * 6 for s in s2]     # one-launch path, per linear
    bytes2 = sum(bytes1)
    del sets
    return {"bert_base_layer_b1_s128_us": fused_us, "bert_base_layer_b1_s128_cold_us": cold_us,
            "bert_base_layer_b1_s128_two_call_us": us, "bert_base_layer_b1_s128_two_call_graph_us": graph_us,
            "eight_minimal_launches_us": floor_us,
            "kernel_us": {s.name: t for s, t in zip(s2, kernel_us)},
            "kernel_GBps_warm": {s.name: b_ / (t * 1e-6) / 1e9 for s, b_, t in zip(s2, bytes1, kernel_us)},
            "algorithmic_bytes": bytes2,
            "achieved_GBps_warm": bytes2 / (fused_us * 1e-6) / 1e9,
            "achieved_GBps_cold": bytes2 / (cold_us * 1e-6) / 1e9,
            "cold_working_set_MB": bytes2 * cold_sets / 2 ** 20,
            "note": "bert_base_layer_b1_s128_us: 4 x w4a4_linear_f16act (quantize_act inside the GEMM kernel, "
                    "one launch per linear, outputs identical to the two-call path), back-to-back layers on one set of "
                    "operands (warm: weights stay in cache); ..._cold_us: the same four launches over 96 rotating sets of "
                    "operands and outputs, every byte from HBM; two_call: 4 x (quantize_act + w4a4_linear), eager and "
                    "replayed from a HIP graph; kernel_us: kernel-boundary durations of the four one-launch kernels; "
                    "attention, LayerNorm and residuals are outside the path; eight_minimal_launches_us = eight "
                    "one-token quantize_act launches, the launch floor of eight launches on this stream"}


# ------------------------------------------------------------------------------------------ token-wise quantizer alone
def quantize_leg(specs, layout, settle_ms, nset=8):
    """w4a4_quantize_act alone at the shapes of the workload, over `nset` rotating inputs (so that nothing is served
    from cache): HBM-bound, read 2 bytes and write half a byte per element."""
    import torch
    from paper_2301_12017_amd import binding as B
    out = {}
    gen = torch.Generator(device="cuda").manual_seed(3)
    for M, K in sorted({(s.M, s.K) for s in specs}):
        xs = [torch.randn((M, K), device="cuda", generator=gen).half() for _ in range(nset)]
        calls = [B.PreparedQuantizeAct(x, B._new_qact(M, K, specs[0].mode, specs[0].group, layout, x.device)) for x in xs]
        st = B._stream()
        settle(lambda: [c(st) for c in calls], min(settle_ms, 50.0))
        reps = 25
        t0 = time.perf_counter()
        for _ in range(reps):
            for c in calls:
                c(st)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / (reps * nset)
        ng = 1 if specs[0].group == 0 else K // specs[0].group
        nbytes = M * K * 2 + M * K // 2 + M * (8 + (4 * ng if specs[0].mode else 0))
        out[f"{M}x{K}"] = {"us": us, "algorithmic_bytes": nbytes, "GBps": nbytes / (us * 1e-6) / 1e9,
                           "frac_of_hbm_peak": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
        del xs, calls
    out["note"] = "back-to-back launches over eight rotating inputs, launch gaps included; fp16 in, packed codes + scales out"
    return out


def copy_probe(mb):
    import torch
    src = torch.empty(mb << 20, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the path is token-parallel with no "
              "exchange); --gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)
    # the CPU oracle first: its worker processes are forked, which must happen before this process touches the GPU
    cpu = None
    plain_step = not (args.gemm_curve or args.latency_only or args.quantize_only or args.config == 5)
    if plain_step and not args.no_cpu_baseline and not args.step_only:
        cpu = cpu_baseline(args.config, args.cpu_rows)
    if args.gemm_curve:
        return bench_curve(args)
    if args.config == 5:
        return bench_chain(args)
    import torch
    from paper_2301_12017_amd import binding as B, workloads as WL
    B.lib()
    torch.cuda.set_device(0)
    if args.latency_only:
        lat = latency_leg(args.settle_ms)
        if args.copy_probe_mb:
            copy_probe(args.copy_probe_mb)
        print(json.dumps({"metric": "BERT-base layer linears latency b1/s128", "unit": "us", "n_gpus": 1, "data": "synthetic",
                          "latency": lat}))
        return
    cfg = args.config
    wl = StepWorkload(cfg, args.schedule, args.layout)
    specs, layers, Xs, outs, stream, schedules = wl.specs, wl.layers, wl.Xs, wl.outs, wl.stream, list(wl.schedules)
    all_fp6 = all(l_.W.layout == B.LAYOUT_FP6 for l_ in layers)
    if args.quantize_only:
        q = quantize_leg(specs, layers[0].W.layout, args.settle_ms)
        if args.copy_probe_mb:
            copy_probe(args.copy_probe_mb)
        print(json.dumps({"metric": "w4a4_quantize_act alone", "unit": "GB/s", "n_gpus": 1, "data": "synthetic", "quantize_act": q}))
        return
    side_legs = cfg == 3 and not args.step_only
    r = wl.measure(args.steps, args.warmup, args.settle_ms)
    ms_per_step, tops, gemm_ms, achieved, ops = r["ms_per_step"], r["TOPS"], r["gemm_ms"], r["achieved_TOPS"], wl.ops
    step = wl.step

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

    lat = latency_leg(args.settle_ms) if side_legs else {}
    lat_settle = min(args.settle_ms, 50.0)
    side_steps = min(args.steps, 50)                              # the side legs are context: shorter timed regions

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

    # ---- the token-wise quantizer alone, and producer fusion (Sec. 4.2): LayerNorm(x + residual) fused with the
    # token-wise quantize, at the hidden size of this workload; HBM-bound, so both are reported against the HBM peak.
    # Rotating buffer sets (> the 256 MB on-package cache) so that nothing is served from cache.
    ln, qleg = {}, {}
    if side_legs:
        qleg = quantize_leg(specs, layers[0].W.layout, args.settle_ms)
        Mh, Kh, nset = specs[0].M, specs[0].K, 4
        rng_t = torch.Generator(device="cuda").manual_seed(0)
        sets = []
        for _ in range(nset):
            x = torch.randn((Mh, Kh), device="cuda", generator=rng_t).half()
            r_ = torch.randn((Mh, Kh), device="cuda", generator=rng_t).half()
            g = (1.0 + 0.1 * torch.randn((Kh,), device="cuda", generator=rng_t)).half()
            b = (0.1 * torch.randn((Kh,), device="cuda", generator=rng_t)).half()
            out = B._new_qact(Mh, Kh, B.SYM, 0, layers[0].W.layout, x.device)
            y = torch.empty((Mh, Kh), dtype=torch.float16, device="cuda")
            sets.append(B.PreparedLayerNormQuantize(x, r_, g, b, 1e-12, out, y))
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
        del sets

    # ---- the INT8 sibling on the same workload (the paper's Sec. 4.1 comparison, on this hardware): the same
    # step with w8a8_quantize_rows + w8a8_linear, timed the same way
    i8 = {}
    if side_legs:
        w8 = [B.quantize_rows8(WL.dev(WL.make_layer(s_, cfg, i, keep_host=True).host_W)) for i, s_ in enumerate(specs)]
        a8 = [B.quantize_rows8(X) for X in Xs]
        q8_calls = [B.PreparedQuantizeRows8(X, a[0], a[1]) for X, a in zip(Xs, a8)]
        l8_calls = [B.PreparedLinear8(a[0], a[1], w[0], w[1], L.bias, L.act, out=o[0])
                    for a, w, L, o in zip(a8, w8, layers, outs)]
        t8 = [[B.KernelTimer() for _ in specs] for _ in range(side_steps)]

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
        for _ in range(side_steps):
            step8()
        torch.cuda.synchronize()
        ms8 = (time.perf_counter() - t6) * 1e3 / side_steps
        for k in range(side_steps):
            step8(t8[k])
        torch.cuda.synchronize()
        g8 = [sum(t8[k][i].elapsed_ms() for k in range(side_steps)) / side_steps for i in range(len(specs))]
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
            for _ in range(side_steps):
                for X, W_, Y_ in zip(Xs, Wh, Yh):
                    torch.matmul(X, W_.t(), out=Y_)
            torch.cuda.synchronize()
            ms16 = (time.perf_counter() - t7) * 1e3 / side_steps
            fp16 = {"ms_per_step": ms16, "TFLOPS": ops / (ms16 * 1e-3) / 1e12,
                    "w4a4_step_speedup": ms16 / ms_per_step,
                    "note": "four torch.matmul calls (hipBLASLt FP16, fp32 accumulate) on the same activations and "
                            "shapes, launch gaps included; the W4A4 step it is compared with also contains the four "
                            "quantize_act kernels, bias and GELU"}
            del Wh, Yh
        except Exception as ex:                                   # context only: never fail the bench over it
            fp16 = {"error": str(ex)}
        try:                                                          # and its INT8 GEMM (int32 out, no epilogue)
            a8l = [a[0] for a in a8]
            w8l = [w[0].t() for w in w8]
            settle(lambda: [torch._int_mm(a_, w_) for a_, w_ in zip(a8l, w8l)], args.settle_ms)
            t8l = time.perf_counter()
            for _ in range(side_steps):
                for a_, w_ in zip(a8l, w8l):
                    torch._int_mm(a_, w_)
            torch.cuda.synchronize()
            ms8l = (time.perf_counter() - t8l) * 1e3 / side_steps
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

    # ---- measured ceilings, and the other two large workloads under this run's clock (short legs)
    ceil, other = {}, {}
    if side_legs:
        ceil = ceilings_leg(args.settle_ms)
        del wl, layers, Xs, outs, step
        torch.cuda.empty_cache()
        w4 = StepWorkload(4)
        r4 = w4.measure(5, 2, args.settle_ms)
        other["cfg4"] = {"workload": "configs[3]: asymmetric INT4, weight groups of 128, M=16384, BERT-base shapes; "
                                     "quantize_act + w4a4_linear x 4",
                         "steps": 5, "ms_per_step": r4["ms_per_step"], "TOPS": r4["TOPS"],
                         "kernel_ms": r4["kernel_ms_per_step"], "frac": r4["achieved_TOPS"] / INT8_MFMA_PEAK_TOPS,
                         "per_gemm_ms": {s_.name: t for s_, t in zip(w4.specs, r4["gemm_ms"])},
                         "kernel": kernel_label(w4.schedules)}
        del w4
        torch.cuda.empty_cache()
        r5 = chain_leg(5, 2, args.settle_ms)
        other["cfg5"] = {"workload": "configs[4]: one layer of the chained BERT-large stack, M=32768, every output "
                                     "requantized in the GEMM epilogue; 4 x w4a4_linear(requant)",
                         "steps": 5, "ms_per_step": r5["ms_per_step"], "TOPS": r5["TOPS"],
                         "kernel_ms": r5["kernel_ms_per_step"], "frac": r5["achieved_TOPS"] / INT8_MFMA_PEAK_TOPS,
                         "per_gemm_ms": dict(zip(r5["names"], r5["gemm_ms"])),
                         "kernel": "gemm_olay_kernel with the fused requantize epilogue; schedules " + ", ".join(r5["schedules"])}
        # the same chained layer with every operand and every requantized output in the FP6 operand layout: the GEMMs run
        # on the FP6 matrix instruction and write the next GEMM's operand themselves (3/4 byte per output)
        torch.cuda.empty_cache()
        r56 = chain_leg(5, 2, args.settle_ms, B.LAYOUT_FP6)
        other["cfg5_fp6_path"] = {"workload": "configs[4] again, every GEMM on the FP6 matrix instruction, every output requantized "
                                              "in its epilogue into the FP6 operand layout; 4 x w4a4_linear(requant)",
                                  "steps": 5, "ms_per_step": r56["ms_per_step"], "TOPS": r56["TOPS"],
                                  "step_speedup_over_int8_path": r5["ms_per_step"] / r56["ms_per_step"],
                                  "kernel_ms": r56["kernel_ms_per_step"],
                                  "frac_of_int8_mfma_peak": r56["achieved_TOPS"] / INT8_MFMA_PEAK_TOPS,
                                  "frac_of_fp6_mfma_peak": r56["achieved_TOPS"] / FP6_MFMA_PEAK_TOPS,
                                  "per_gemm_ms": dict(zip(r56["names"], r56["gemm_ms"])),
                                  "kernel": "gemm_fp6_kernel with the fused requantize epilogue; schedules " + ", ".join(r56["schedules"])}

        if cfg == 3:
            # the same step with the layers of at least 2M weights in the FP6 operand layout: their GEMMs run on the FP6
            # matrix instruction (exact integer sums in its FP32 accumulator); the others stay on the int8 MFMA
            torch.cuda.empty_cache()
            lay6 = [B.LAYOUT_FP6 if s_.N * s_.K >= (1 << 21) else B.LAYOUT_MFMA for s_ in specs]
            w6 = StepWorkload(3, 0, lay6)
            r6 = w6.measure(side_steps, args.warmup, args.settle_ms)
            ops6 = sum(2 * s_.M * s_.N * s_.K for s_, l_ in zip(specs, lay6) if l_ == B.LAYOUT_FP6)
            ms6 = sum(t for t, l_ in zip(r6["gemm_ms"], lay6) if l_ == B.LAYOUT_FP6)
            other["cfg3_fp6_path"] = {
                "workload": "configs[2] again, " + ", ".join(s_.name for s_, l_ in zip(specs, lay6) if l_ == B.LAYOUT_FP6)
                            + " in the FP6 operand layout (v_mfma_f32_32x32x64_f8f6f4, FP6 E2M3 x FP6 E2M3 -> FP32, exact for "
                              "symmetric INT4 codes), the rest on the int8 MFMA; quantize_act + w4a4_linear x 4",
                "steps": side_steps, "ms_per_step": r6["ms_per_step"], "TOPS": r6["TOPS"],
                "step_speedup_over_int8_path": ms_per_step / r6["ms_per_step"],
                "kernel_ms": r6["kernel_ms_per_step"], "kernel_TOPS": r6["achieved_TOPS"],
                "frac_of_int8_mfma_peak": r6["achieved_TOPS"] / INT8_MFMA_PEAK_TOPS,
                "fp6_kernels": {"ops": ops6, "ms": ms6, "TOPS": ops6 / (ms6 * 1e-3) / 1e12,
                                "frac_of_fp6_mfma_peak": ops6 / (ms6 * 1e-3) / 1e12 / FP6_MFMA_PEAK_TOPS,
                                "frac_of_measured_fp6": ops6 / (ms6 * 1e-3) / 1e12 / ceil["mfma_fp6_int4_codes_TOPS"]},
                "per_gemm_ms": {s_.name: t for s_, t in zip(w6.specs, r6["gemm_ms"])},
                "kernel": kernel_label(w6.schedules)}
            del w6

    roof = {"bound": "mfma", "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
            "frac": achieved / INT8_MFMA_PEAK_TOPS,
            "traffic": profiled_traffic(schedules) if cfg == 3 else None,
            "traffic_unit": "HBM-side bytes per step (the four launches), from the rocprofv3 --pmc summary "
                            "profiles/gemm_config3_hbm_traffic.txt when it was taken on these schedules, else null",
            "kernel": kernel_label(schedules), "ops_per_step": ops, "kernel_ms_per_step": sum(gemm_ms)}
    if ceil:
        roof["measured_peak"] = ceil["mfma_int4_codes_TOPS"]
        roof["frac_of_measured"] = achieved / ceil["mfma_int4_codes_TOPS"]
    line = {
        "metric": METRIC,
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_ms": args.settle_ms,
        "ms_per_step": ms_per_step, "ms_per_step_graph_replay": graph_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": (DTYPE_FP6 if all_fp6 else DTYPE).format("fp16"),
        "data": "synthetic",
        "config": {"workload": f"configs[{cfg - 1}]: " + ", ".join(f"{s.name} {s.M}x{s.N}x{s.K}" for s in specs)
                   + ("; symmetric per-token / per-channel INT4" if cfg != 4 else
                      "; asymmetric INT4, weight groups of 128, 8 outlier channels x20"),
                   "step": "quantize_act + w4a4_linear (fused GEMM, dequant, bias, GELU on ffn1, fp16 store) x 4",
                   "schedule": args.schedule},
        "pct_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
        "per_gemm": [{"name": s.name, "ms": t, "TOPS": 2 * s.M * s.N * s.K / (t * 1e-3) / 1e12,
                      "frac": 2 * s.M * s.N * s.K / (t * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, "schedule": n}
                     for s, t, n in zip(specs, gemm_ms, schedules)],
        "latency": lat,
        "whole_layer_b1_s128": whole,
        "quantize_act": qleg,
        "producer_fusion": ln,
        "int8_sibling": i8,
        "per_part_strategy": strat,
        "fp16_library_gemm": fp16,
        "ceilings": ceil,
        "other_workloads": other,
        "roofline": roof,
        "consistency": {"timed_region_s": r["timed_region_s"]},
    }
    if args.copy_probe_mb:
        copy_probe(args.copy_probe_mb)
    if cpu is not None:
        line["cpu_baseline"] = cpu
    print(json.dumps(line))


def bench_curve(args):
    """Sec. 4.1 compares the INT4 with the INT8 GEMM over the token count M for the four encoder shapes.  Here: the
    fused linears (GEMM + dequantize + fp16 store, operands already quantized), kernel-boundary times."""
    import torch
    from paper_2301_12017_amd import binding as B, synth
    B.lib()
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda").manual_seed(0)
    reps = max(min(args.steps, 20), 5)
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


if __name__ == "__main__":
    main()
