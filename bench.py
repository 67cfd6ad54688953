#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

Workload (default): the Llama-7B-shaped decode stack at batch 1 -- 32 layers x
{q,k,v,o 4096x4096; gate,up 4096->11008; down 11008->4096}, group-128 int4 and
int8 copies of every weight resident in HBM, the bit-width of every linear drawn
per token from {4, 8} with p = 1/2 (seeded, 128 distinct patterns), and one
entropy + KL reduction over a 32000-entry logits pair per token.  One *step* =
one token = all 224 linears in the order a decoder must issue them (q/k/v, o,
gate/up, down, layer after layer: 128 dependent stages in ONE launch of the
stage-ordered plan, per-entry bit-widths read from device memory) followed by
one fq_entropy_kl launch.  The same linears as one plan of independent entries
are timed beside it (`independent_order`).  Attention, norms,
embeddings, lm_head, sampling and the KV cache are not part of the path.

Every tensor is synthetic and seeded (module ``synth``); weights are quantized
on the GPU by fq_quantize.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import synth  # noqa: E402

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
# HBM bytes per plan launch of the default workload relative to its algorithmic bytes, measured
# with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB copy
# (profiles/decode_m1_plan_llama7b_hbm_traffic.md); reported only for that workload.
MEASURED_TRAFFIC_RATIO = {("llama7b", 1, (4, 8)): 4993151.0 / 4978290.0,
                          ("llama7b", 1, (4, 8), "dependent"): 5040493.0 / 4978290.0,
                          ("llama7b", 16, (4, 8, 16)): 8.052 / 7.857}
# where those ratios come from (a constant carried from a profile, not counters read in this run)
TRAFFIC_SOURCE = {("llama7b", 1, (4, 8)): "profiles/decode_m1_plan_llama7b_hbm_traffic.md (rocprofv3 --pmc, scaled by a 1 GiB copy)",
                  ("llama7b", 1, (4, 8), "dependent"): "profiles/decode_staged_plan_llama7b_hbm_traffic.md (rocprofv3 --pmc, scaled by a 1 GiB read)",
                  ("llama7b", 16, (4, 8, 16)): "profiles/decode_stream_plan_llama7b_batch16_kernel_trace.md (rocprofv3 --pmc)"}
N_PATTERNS = 128        # decode steps with distinct per-layer bit patterns
VOCAB = 32000
SEED = 0


def weight_bytes(N: int, K: int, bits: int) -> int:
    """Bytes a call must read for its weights: packed codes + fp32 scale + u8 zero per
    group of 128 (bits = 16: the fp16 matrix)."""
    if bits == 16:
        return 2 * N * K
    return N * K * bits // 8 + (N * K // 128) * 5


class Stack:
    """The resident multi-precision weight store of one synthetic model and a plan over it."""

    def __init__(self, name: str, M: int = 1, bit_choices=(4, 8), layers: int | None = None,
                 verbose: bool = False):
        import torch
        import paper_2506_12024_amd as fq

        self.fq, self.torch = fq, torch
        dev = "cuda:0"
        n_layers, hidden, ffn, std, outl = synth.STACKS[name]
        if layers is not None:
            n_layers = layers
        self.name, self.M, self.bit_choices = name, M, tuple(bit_choices)
        self.std, self.outl = std, outl
        self.entries = []   # (layer index, matrix name, K, N)
        self.layers, self.xs, self.ys, self.keep = [], [], [], []
        t0 = time.time()
        for li in range(n_layers):
            for mname, K, N in synth.llama_linears(hidden, ffn, synth.KV_WIDTH.get(name)):
                w = synth.weight(SEED, self.wname(li, mname), N, K, std, outlier_p=outl)
                w_dev = torch.from_numpy(w.view(np.int16)).to(dev).view(torch.float16)
                layer = fq.Layer(N, K)
                for b in self.bit_choices:
                    if b == 16:
                        layer.attach(16, w_dev)
                        self.keep.append(w_dev)
                        continue
                    cb, sb, zb = fq.fq_packed_sizes(N, K, b)
                    codes = torch.empty(cb, dtype=torch.uint8, device=dev)
                    scales = torch.empty(sb // 4, dtype=torch.float32, device=dev)
                    zeros = torch.empty(zb, dtype=torch.uint8, device=dev)
                    fq.fq_quantize(w_dev, N, K, b, 128, codes, scales, zeros)
                    layer.attach(b, codes, scales, zeros)
                x = synth.activations(SEED, self.xname(li, mname), M, K)
                self.xs.append(torch.from_numpy(x.view(np.int16)).to(dev).view(torch.float16))
                self.ys.append(torch.zeros((M, N), dtype=torch.float16, device=dev))
                self.layers.append(layer)
                self.entries.append((li, mname, K, N))
            if verbose:
                print("  built layer %d/%d (%.1f s)" % (li + 1, n_layers, time.time() - t0),
                      file=sys.stderr, flush=True)
        torch.cuda.synchronize()
        n = len(self.layers)
        self.workspace = torch.empty(fq.Plan.workspace_bytes(n), dtype=torch.uint8, device=dev)
        self.plan = fq.Plan(self.layers, self.xs, self.ys, M, self.workspace)
        # per-token bit-width patterns, drawn on the host before timing
        pats = np.stack([synth.choice(SEED, "%s/bits/step%d" % (name, s), n, self.bit_choices)
                         for s in range(N_PATTERNS)])
        self.patterns = pats
        self.bits_dev = torch.from_numpy(pats).to(dev)
        # logits pair per step
        a, b = synth.logits_pair(SEED, "%s/logits" % name, N_PATTERNS * M, VOCAB)
        self.logits_a = torch.from_numpy(a).to(dev)
        self.logits_b = torch.from_numpy(b).to(dev)
        self.logits_host = (a, b)
        self.H = torch.zeros((N_PATTERNS, M), dtype=torch.float32, device=dev)
        self.KL = torch.zeros((N_PATTERNS, M), dtype=torch.float32, device=dev)
        self.build_seconds = time.time() - t0

    def wname(self, li, mname):
        return "%s/L%d/%s/w" % (self.name, li, mname)

    def xname(self, li, mname):
        return "%s/L%d/%s/x/M%d" % (self.name, li, mname, self.M)

    def step_bytes(self, s: int) -> int:
        return sum(weight_bytes(N, K, int(b)) for (_, _, K, N), b in zip(self.entries, self.patterns[s % N_PATTERNS]))

    def run_linears(self, s: int):
        self.plan.run(self.bits_dev[s % N_PATTERNS])

    def run_entropy(self, s: int):
        i, M = s % N_PATTERNS, self.M
        self.fq.fq_entropy_kl(self.logits_a[i * M:(i + 1) * M], self.logits_b[i * M:(i + 1) * M], M, VOCAB,
                              self.H[i], self.KL[i])

    def step(self, s: int):
        self.run_linears(s)
        self.run_entropy(s)

    def build_stage_plans(self):
        """Four plans per decoder layer (q/k/v, o, gate/up, down): the grouping a real decoder
        allows, where only linears that share an input are independent of each other."""
        torch, fq = self.torch, self.fq
        groups = {"q": 0, "k": 0, "v": 0, "o": 1, "gate": 2, "up": 2, "down": 3}
        stages = {}
        for e, (li, mname, _, _) in enumerate(self.entries):
            stages.setdefault((li, groups[mname]), []).append(e)
        self.stage_plans = []
        for key in sorted(stages):
            idx = stages[key]
            ws = torch.empty(fq.Plan.workspace_bytes(len(idx)), dtype=torch.uint8, device="cuda:0")
            plan = fq.Plan([self.layers[i] for i in idx], [self.xs[i] for i in idx],
                           [self.ys[i] for i in idx], self.M, ws)
            self.stage_plans.append((plan, idx[0], len(idx)))

    def build_staged_plan(self):
        """The same stages in ONE stage-ordered plan: a single persistent launch walks them in order."""
        torch, fq = self.torch, self.fq
        groups = {"q": 0, "k": 0, "v": 0, "o": 1, "gate": 2, "up": 2, "down": 3}
        stage = [4 * li + groups[mname] for (li, mname, _, _) in self.entries]
        assert all(b >= a for a, b in zip(stage, stage[1:])), "entries are listed in stage order"
        self.staged_ws = torch.empty(fq.StagedPlan.workspace_bytes(len(stage), max(stage) + 1), dtype=torch.uint8,
                                     device="cuda:0")
        self.staged_plan = fq.StagedPlan(self.layers, self.xs, self.ys, stage, self.M, self.staged_ws)
        self.n_stages = max(stage) + 1

    def run_linears_one_launch_staged(self, s: int):
        self.staged_plan.run(self.bits_dev[s % N_PATTERNS])

    def run_linears_staged(self, s: int):
        bits = self.bits_dev[s % N_PATTERNS]
        for plan, first, n in self.stage_plans:
            plan.run(bits[first:first + n])


def dependent_order_as_launches(stack: "Stack", W: int, K_steps: int) -> dict:
    """The dependent order as separate launches: 4 plan launches per decoder layer (q/k/v, o, gate/up,
    down), captured once in a HIP graph and replayed; milliseconds per step."""
    import torch
    stack.build_stage_plans()
    stack.run_linears_staged(W)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        stack.run_linears_staged(W)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            stack.run_linears_staged(W)
    torch.cuda.synchronize()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = max(8, K_steps // 4)
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    return {"dependent_order_as_%d_launches_ms" % len(stack.stage_plans): ms,
            "dependent_order_as_launches_tokens_per_s": stack.M * 1e3 / ms}


def _set_omp_threads(n: int) -> bool:
    """Number of threads of the OpenMP runtime the oracle's library runs on (the oracle itself is
    untouched: this is the call OMP_NUM_THREADS would make at start-up)."""
    import ctypes
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except OSError:
        return False


def _oracle_step_seconds(stack: Stack, sample_layers: int):
    """Seconds the oracle takes for the linears of the first `sample_layers` decoder layers of step
    0 (weights regenerated from the same seeds and quantized by the oracle at the drawn bit-width
    before the clock starts) and for the step's entropy/KL."""
    import oracle

    prepared = []
    for (li, mname, K, N), b in zip(stack.entries, stack.patterns[0]):
        if li >= sample_layers:
            break
        w = synth.weight(SEED, stack.wname(li, mname), N, K, stack.std, outlier_p=stack.outl)
        x = synth.activations(SEED, stack.xname(li, mname), stack.M, K)
        b = int(b)
        packed = (w, None, None) if b == 16 else oracle.quantize(w, b)
        prepared.append((x, packed, b))
    a, bl = stack.logits_host
    M = stack.M
    t0 = time.perf_counter()
    for x, (c, s, z), b in prepared:
        oracle.linear(x, c, s, z, b)
    t_lin = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.entropy_kl(a[:M], bl[:M])
    t_ent = time.perf_counter() - t0
    return t_lin, t_ent


def cpu_baseline(stack: Stack, sample_layers: int = 8) -> dict:
    """The CPU oracle, as it stands, on a bounded sample of the same workload, scaled to the whole
    stack: on all the host threads it is given (its OpenMP loops run over output rows) and on one
    thread (a smaller sample)."""
    n_layers = synth.STACKS[stack.name][0]
    sample_layers = min(sample_layers, n_layers)
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    M = stack.M
    t_lin, t_ent = _oracle_step_seconds(stack, sample_layers)
    t_step = t_lin * (n_layers / sample_layers) + t_ent
    out = {"value": M / t_step, "unit": "tokens/s", "cores": threads, "kind": "oracle",
           "sample": "step 0: linears of the first %d of %d decoder layers (%.2f s on %d threads = %.0f core-seconds, "
                     "scaled x%.0f) + entropy/KL of the step's logits (%.4f s)"
                     % (sample_layers, n_layers, t_lin, threads, t_lin * threads, n_layers / sample_layers, t_ent)}
    if threads > 1 and _set_omp_threads(1):
        one = max(1, sample_layers // 8)
        t_lin1, t_ent1 = _oracle_step_seconds(stack, one)
        _set_omp_threads(threads)
        out["single_thread"] = {"value": M / (t_lin1 * (n_layers / one) + t_ent1), "unit": "tokens/s", "cores": 1,
                                "sample": "step 0: linears of the first %d of %d decoder layers (%.2f s on one thread, "
                                          "scaled x%.0f) + entropy/KL (%.4f s)"
                                          % (one, n_layers, t_lin1, n_layers / one, t_ent1)}
    return out


def bench_prefill(args):
    """The prefill-shaped slice: x[2048][8192] against W 8192->28672 and x[2048][28672] against
    W 28672->8192 (a 70B-shaped layer slice), int4 and int8, MFMA dequant-GEMM.  One step = the
    GEMMs of the chosen shapes (`--shape NxK`, default both) and bit-widths (`--prefill-bits`,
    default 4,8; 2 and 16 are served too).  Reports TFLOP/s against the dense fp16 MFMA peak, per
    call and as the mean."""
    import torch
    import paper_2506_12024_amd as fq
    dev, M = "cuda:0", 2048
    shapes = [(28672, 8192), (8192, 28672)]
    if args.shape:
        shapes = [tuple(int(v) for v in args.shape.lower().split("x"))]
    widths = [int(b) for b in args.prefill_bits.split(",")]
    calls = []
    for N, K in shapes:
        w = synth.weight(SEED, "prefill/%dx%d/w" % (N, K), N, K, 0.015)
        x = synth.activations(SEED, "prefill/%dx%d/x" % (N, K), M, K)
        w_dev = torch.from_numpy(w.view(np.int16)).to(dev).view(torch.float16)
        x_dev = torch.from_numpy(x.view(np.int16)).to(dev).view(torch.float16)
        y = torch.empty((M, N), dtype=torch.float16, device=dev)
        layer = fq.Layer(N, K)
        for b in widths:
            if b == 16:
                layer.attach(16, w_dev)
            else:
                cb, sb, zb = fq.fq_packed_sizes(N, K, b)
                c = torch.empty(cb, dtype=torch.uint8, device=dev)
                sc = torch.empty(sb // 4, dtype=torch.float32, device=dev)
                z = torch.empty(zb, dtype=torch.uint8, device=dev)
                fq.fq_quantize(w_dev, N, K, b, 128, c, sc, z)
                layer.attach(b, c, sc, z)
            calls.append((layer, b, x_dev, y))
        if 16 not in widths:
            del w_dev
    flop = sum(2.0 * M * l.N * l.K for l, _, _, _ in calls)

    def step():
        for layer, b, x_dev, y in calls:
            fq.fq_linear(layer, b, x_dev, M, y)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_launch = e0.elapsed_time(e1) / (args.steps * len(calls))
    achieved = flop / len(calls) / (ms_launch * 1e-3) / 1e12
    per_call = {}
    for layer, b, x_dev, y in calls:   # each GEMM by itself, back to back
        e0.record(stream)
        for _ in range(10):
            fq.fq_linear(layer, b, x_dev, M, y)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        per_call["%d->%d W%d" % (layer.K, layer.N, b)] = {"ms": ms, "TFLOPs": 2.0 * M * layer.N * layer.K / (ms * 1e-3) / 1e12}
    print(json.dumps({
        "metric": "prefill dequant-GEMM throughput", "value": M * args.steps * len(calls) / elapsed,
        "unit": "tokens*layers/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "70B-shaped slice: M=2048, %s, W%s (%d GEMMs per step)"
                               % (" and ".join("%d->%d" % (K, N) for N, K in shapes),
                                  "/W".join(str(b) for b in widths), len(calls))},
        "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": achieved, "peak": 2500.0,
                     "unit": "TFLOP/s", "frac": achieved / 2500.0, "traffic": None,
                     "avg_launch_ms": ms_launch, "flop_per_launch": flop / len(calls)},
        "per_call": per_call}))


def bench_prefill_w8a8(args):
    """The same 70B-shaped slice in the paper's own prefill arithmetic (Sec. 4.3: W8A8 on the
    integer matrix units): per step, each of the two GEMMs quantizes its activations per token
    (fq_quantize_act) and multiplies them by the resident INT8 weights (fq_linear_w8a8).  Reports
    TOP/s of the GEMM kernel against the dense int8 MFMA peak."""
    import torch
    import paper_2506_12024_amd as fq
    dev, M = "cuda:0", 2048
    calls = []
    shapes = [(28672, 8192), (8192, 28672)]
    if args.shape:
        shapes = [tuple(int(v) for v in args.shape.lower().split("x"))]
    for N, K in shapes:
        w = synth.weight(SEED, "prefill/%dx%d/w" % (N, K), N, K, 0.015)
        x = synth.activations(SEED, "prefill/%dx%d/x" % (N, K), M, K)
        w_dev = torch.from_numpy(w.view(np.int16)).to(dev).view(torch.float16)
        x_dev = torch.from_numpy(x.view(np.int16)).to(dev).view(torch.float16)
        group = K if args.w8a8_group == "row" else 128
        layer = fq.Layer(N, K, group)
        cb, sb, zb = fq.fq_packed_sizes(N, K, 8, group)
        c = torch.empty(cb, dtype=torch.uint8, device=dev)
        sc = torch.empty(sb // 4, dtype=torch.float32, device=dev)
        z = torch.empty(zb, dtype=torch.uint8, device=dev)
        fq.fq_quantize(w_dev, N, K, 8, group, c, sc, z)
        layer.attach(8, c, sc, z)
        del w_dev
        calls.append((layer, x_dev, torch.empty((M, K), dtype=torch.int8, device=dev),
                      torch.empty(M, dtype=torch.float32, device=dev),
                      torch.empty((K // 128, M), dtype=torch.int32, device=dev),
                      torch.empty((M, N), dtype=torch.float16, device=dev)))
    ops = sum(2.0 * M * l.N * l.K for l, *_ in calls)

    def step(gemm=True, quant=True):
        for layer, x_dev, xq, sx, xsum, y in calls:
            if quant:
                fq.fq_quantize_act(x_dev, M, layer.K, xq, sx, xsum)
            if gemm:
                fq.fq_linear_w8a8(layer, xq, sx, xsum, M, y)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    e0.record(stream)
    for _ in range(args.steps):
        step(quant=False)
    e1.record(stream)
    torch.cuda.synchronize()
    ms_launch = e0.elapsed_time(e1) / (args.steps * len(calls))
    e0.record(stream)
    for _ in range(args.steps):
        step(gemm=False)
    e1.record(stream)
    torch.cuda.synchronize()
    ms_quant = e0.elapsed_time(e1) / (args.steps * len(calls))
    achieved = ops / len(calls) / (ms_launch * 1e-3) / 1e12
    print(json.dumps({
        "metric": "W8A8 prefill GEMM throughput", "value": M * args.steps * len(calls) / elapsed,
        "unit": "tokens*layers/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "70B-shaped slice: M=2048, 8192->28672 and 28672->8192, per-token int8 "
                               "activations x %s INT8 weights (2 quantize + 2 GEMM launches per step)"
                               % ("one-scale-per-row" if args.w8a8_group == "row" else "group-128")},
        "roofline": {"bound": "mfma", "kernel": "w8a8_row_kernel" if args.w8a8_group == "row" else "w8a8_kernel", "achieved": achieved, "peak": 5000.0,
                     "unit": "TOP/s", "frac": achieved / 5000.0, "traffic": None,
                     "avg_launch_ms": ms_launch, "ops_per_launch": ops / len(calls)},
        "quantize_act_avg_launch_ms": ms_quant}))


def kl_replacement_order(stack):
    """The offline analysis of Sec. 3.1 / 4.3, mechanics only (synthetic weights carry no
    meaning): every linear runs once at INT8 and once at INT4 on its own seeded input, the KL
    divergence between softmax of the two outputs is reduced per row by fq_entropy_kl_f16, and
    fq_rank_ascending sorts the linears by it -- smaller KL is replaced first.  Everything stays
    on the device; returns (order int32 [n], kl f32 [n][M])."""
    import torch
    fq = stack.fq
    dev, n, M = "cuda:0", len(stack.layers), stack.M
    ys4 = [torch.empty_like(y) for y in stack.ys]
    ws = torch.empty(fq.Plan.workspace_bytes(n), dtype=torch.uint8, device=dev)
    plan4 = fq.Plan(stack.layers, stack.xs, ys4, M, ws)
    stack.plan.run(torch.full((n,), 8, dtype=torch.int32, device=dev))
    plan4.run(torch.full((n,), 4, dtype=torch.int32, device=dev))
    kl = torch.empty((n, M), dtype=torch.float32, device=dev)
    h = torch.empty(M, dtype=torch.float32, device=dev)
    for e, (_, _, _, N) in enumerate(stack.entries):
        fq.fq_entropy_kl_f16(stack.ys[e], ys4[e], M, N, h, kl[e])
    order = torch.empty(n, dtype=torch.int32, device=dev)
    fq.fq_rank_ascending(kl, n, M, order)
    torch.cuda.synchronize()
    return order, kl


def bench_entropy(args):
    """Batched entropy + KL over [2048][128256] fp32 logits pairs (HBM bound: 8 bytes per entry)."""
    import torch
    import paper_2506_12024_amd as fq
    dev, R, V = "cuda:0", 2048, 128256
    a, b = synth.logits_pair(SEED, "entropy/2048x128256", R, V)
    a_dev, b_dev = torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev)
    H = torch.empty(R, device=dev)
    KL = torch.empty(R, device=dev)
    for _ in range(args.warmup):
        fq.fq_entropy_kl(a_dev, b_dev, R, V, H, KL)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        fq.fq_entropy_kl(a_dev, b_dev, R, V, H, KL)
    e1.record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = e0.elapsed_time(e1) / args.steps
    alg = 8.0 * R * V
    achieved = alg / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "batched entropy+KL rows/s", "value": R * args.steps / elapsed, "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "config": {"workload": "entropy + KL over 2048 x 128256 fp32 logits pairs"},
        "roofline": {"bound": "hbm", "kernel": "entropy_kl_kernel", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": None, "avg_launch_ms": ms, "algorithmic_bytes_per_launch": alg}}))


def bench_quantize(args):
    """The quantizers on one 7B-shaped weight (11008 x 4096 fp16): fq_quantize and fq_quantize_sym
    at 4 and 8 bits (read 2 bytes, write bits / 8 + 5 / 128 bytes per weight) and fq_fake_quantize
    at 2 bits (read 2, write 2).  A step is the five calls; the roofline object is the 2-bit
    quantize-dequantize, the others are listed beside it.  HBM bound."""
    import torch
    import paper_2506_12024_amd as fq
    dev, N, K = "cuda:0", 11008, 4096
    w = synth.weight(SEED, "quantize/w", N, K, 0.02, outlier_p=0.001)
    w_dev = torch.from_numpy(w.view(np.int16)).to(dev).view(torch.float16)
    bufs = {}
    for b in (4, 8):
        cb, sb, zb = fq.fq_packed_sizes(N, K, b, 128)
        bufs[b] = (torch.empty(cb, dtype=torch.uint8, device=dev), torch.empty(sb // 4, device=dev),
                   torch.empty(zb, dtype=torch.uint8, device=dev))
    w_hat = torch.empty_like(w_dev)
    calls = [("fq_quantize 4-bit", lambda: fq.fq_quantize(w_dev, N, K, 4, 128, *bufs[4]), 2 + 0.5 + 5 / 128),
             ("fq_quantize 8-bit", lambda: fq.fq_quantize(w_dev, N, K, 8, 128, *bufs[8]), 2 + 1 + 5 / 128),
             ("fq_quantize_sym 4-bit", lambda: fq.fq_quantize_sym(w_dev, N, K, 4, 128, *bufs[4]), 2 + 0.5 + 5 / 128),
             ("fq_quantize_sym 8-bit", lambda: fq.fq_quantize_sym(w_dev, N, K, 8, 128, *bufs[8]), 2 + 1 + 5 / 128),
             ("fq_fake_quantize 2-bit", lambda: fq.fq_fake_quantize(w_dev, N, K, 2, 128, False, w_hat), 4.0)]
    stream = torch.cuda.current_stream()
    per_call = {}
    for name, fn, bytes_per_weight in calls:
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        per_call[name] = {"ms": ms, "GBps": bytes_per_weight * N * K / (ms * 1e-3) / 1e9}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for _, fn, _ in calls:
            fn()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    fake = per_call["fq_fake_quantize 2-bit"]
    out = {
        "metric": "quantizer weights/s (five calls per step)", "value": 5.0 * N * K * args.steps / elapsed,
        "unit": "weights/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "quantizers on one 11008 x 4096 fp16 weight, group 128"},
        "per_call": per_call,
        "roofline": {"bound": "hbm", "kernel": "fake_quantize_kernel", "achieved": fake["GBps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": fake["GBps"] / HBM_PEAK_GBPS, "traffic": None,
                     "avg_launch_ms": fake["ms"], "algorithmic_bytes_per_launch": 4.0 * N * K}}
    if not args.no_cpu_baseline:
        import oracle
        rows = 1024
        t0 = time.perf_counter()
        oracle.fake_quantize(w[:rows], 2)
        oracle.quantize_sym(w[:rows], 4)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * rows * K / dt, "unit": "weights/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                               "sample": "fake_quantize (2-bit) and quantize_sym (4-bit) on the first %d rows" % rows}
    print(json.dumps(out))


def bench_lm_head(args):
    """The output layer of a 7B-shaped model (32000 x 4096 fp16) fused with the entropy and argmax
    of its logits (fq_lm_head_entropy, batch 1), against the same done in two launches through
    fq_linear (fp16 passthrough) and fq_entropy_kl_f16.  HBM bound: 2 bytes per weight."""
    import torch
    import paper_2506_12024_amd as fq
    dev, V, K, M = "cuda:0", VOCAB, 4096, 1
    w = synth.weight(SEED, "lm_head/w", V, K, 0.02)
    x = synth.activations(SEED, "lm_head/x", M, K)
    w_dev = torch.from_numpy(w.view(np.int16)).to(dev).view(torch.float16)
    x_dev = torch.from_numpy(x.view(np.int16)).to(dev).view(torch.float16)
    H = torch.empty(M, device=dev)
    am = torch.empty(M, dtype=torch.int32, device=dev)
    layer = fq.Layer(V, K)
    layer.attach(16, w_dev)
    y = torch.empty((M, V), dtype=torch.float16, device=dev)
    H2 = torch.empty(M, device=dev)

    def fused():
        fq.fq_lm_head_entropy(x_dev, w_dev, M, V, K, None, H, am)

    def separate():
        fq.fq_linear(layer, 16, x_dev, M, y)
        fq.fq_entropy_kl_f16(y, None, M, V, H2, None)

    stream = torch.cuda.current_stream()
    ms = {}
    for name, fn in (("fused", fused), ("separate", separate)):
        for _ in range(args.warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        ms[name] = e0.elapsed_time(e1) / args.steps
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fused()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    alg = 2.0 * V * K
    achieved = alg / (ms["fused"] * 1e-3) / 1e9
    out = {
        "metric": "output layer + entropy + argmax, tokens/s", "value": M * args.steps / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "fp16 output layer 32000 x 4096, batch 1, fused with entropy and argmax"},
        "two_launches_ms": ms["separate"],
        "roofline": {"bound": "hbm", "kernel": "lm_head_entropy_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": None, "avg_launch_ms": ms["fused"],
                     "algorithmic_bytes_per_launch": alg}}
    if not args.no_cpu_baseline:
        import oracle
        rows = 8000
        t0 = time.perf_counter()
        oracle.lm_head_entropy(x, w[:rows])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": M * (rows / V) / dt, "unit": "tokens/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                               "sample": "the first %d of %d vocabulary rows, scaled" % (rows, V)}
    print(json.dumps(out))


def bench_flexquant(args):
    """Alg. 1's decode loop on the 7B-shaped stack over a ladder of resident formats (default FP16 ->
    INT8 -> INT4, the ladder of Sec. 5.1's main setting; `--ladder 8,4` for the two-rung one):
    every linear starts on the first rung; per token the plan runs at the current bit-widths,
    fq_entropy_kl gives the entropy of the token's logits and fq_sched_step (window 20) moves the
    next linears of the replacement order one rung down when the average PPLE falls below the
    threshold -- all on the device, three launches per token.  The replacement order is ascending
    KL between each linear's INT8 and INT4 output, measured once before generation through the
    library (kl_replacement_order); it is walked once per rung.  The logits are synthetic with an
    entropy that falls as generation proceeds (the behaviour Sec. 4.2 reports): one seeded N(0, 1)
    vector scaled by a growing factor."""
    import torch
    import paper_2506_12024_amd as fq
    dev = "cuda:0"
    T = max(args.steps, 64)
    ladder = [int(b) for b in args.ladder.split(",")]
    assert len(ladder) >= 2 and all(b in (2, 3, 4, 8, 16) for b in ladder) and sorted(ladder, reverse=True) == ladder
    widths = tuple(sorted(set(ladder) | {4, 8}))   # 4 and 8 are needed for the KL order
    stack = Stack(args.stack, M=1, bit_choices=widths, layers=args.layers, verbose=args.verbose)
    n = len(stack.layers)
    dependent = args.order != "independent"
    if dependent:
        stack.build_staged_plan()
    plan = stack.staged_plan if dependent else stack.plan
    base = synth.normal_f32(SEED, "flexquant/logits", VOCAB, 1.0)
    scale = (2.0 + 2.0 * np.arange(T, dtype=np.float32) / T)[:, None]
    logits = torch.from_numpy(base[None, :] * scale).to(dev)
    order_dev, kl = kl_replacement_order(stack)
    order = order_dev.cpu().numpy()
    kl_host = kl.cpu().numpy().astype(np.float64).sum(axis=1)
    # the events: the whole order once per step down the ladder
    rungs = len(ladder) - 1
    ev_entry = order_dev.repeat(rungs).contiguous()
    ev_bits = torch.cat([torch.full((n,), b, dtype=torch.int32, device=dev) for b in ladder[1:]]).contiguous()
    n_events = n * rungs
    bits = torch.full((n,), ladder[0], dtype=torch.int32, device=dev)
    ev_token = torch.full((n_events,), -1, dtype=torch.int32, device=dev)
    H = torch.zeros(T, dtype=torch.float32, device=dev)
    state = torch.zeros(fq.fq_sched_state_bytes(20), dtype=torch.uint8, device=dev)
    # a full window of new tokens separates two triggers: size a trigger so that the whole ladder is
    # walked within the run if every window's average stays under the threshold
    per_trigger = -(-n_events // max(1, (T - 1) // 20))

    def generate(sched: bool):
        for t in range(T):
            plan.run(bits)
            fq.fq_entropy_kl(logits[t], None, 1, VOCAB, H[t:t + 1], None)
            if sched:
                fq.fq_sched_step(state, H[t:t + 1])

    # threshold: the mean PPLE of 20 "prefill" positions taken at the start of the run
    generate(False)
    fq.fq_sched_init(state, 20, 0.0, per_trigger, ev_entry, ev_bits, n_events, bits, ev_token)
    fq.fq_sched_threshold_from_prefill(state, H, 20, 20)
    torch.cuda.synchronize()
    results = {}
    for name, start, sched in [("fixed_%d" % b, b, False) for b in ladder] + [("flexquant", ladder[0], True)]:
        bits.fill_(start)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        generate(sched)
        torch.cuda.synchronize()
        results[name] = T / (time.perf_counter() - t0)
    next_event, tokens, thre, last_mean = fq.fq_sched_peek(state)
    tok = ev_token.cpu().numpy().reshape(rungs, n)
    fired = tok[tok >= 0]
    # average bit-width over the generation, weighted by weights per entry: entry order[i] sits on
    # rung r from the token after its r-th event fired
    sizes = np.array([N * K for (_, _, K, N) in stack.entries], dtype=np.float64)
    avg = np.zeros(n)
    for i, e in enumerate(order):
        since = [0] + [int(tok[r, i]) + 1 if tok[r, i] >= 0 else T for r in range(rungs)] + [T]
        avg[e] = sum(ladder[r] * (since[r + 1] - since[r]) for r in range(rungs + 1)) / T
    avg_bits = float((avg * sizes).sum() / sizes.sum())
    status = plan.status()
    out = {
        "metric": "decode tokens/s with on-device precision switching", "value": results["flexquant"],
        "unit": "tokens/s", "n_gpus": 1, "steps": T, "warmup": 0,
        "ms_per_step": 1e3 / results["flexquant"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 x %s -> f32" % "/".join("fp16" if b == 16 else "int%d" % b for b in ladder),
        "data": "synthetic",
        "config": {"workload": "%s stack, batch 1, %s by the PPLE scheduler (window 20, %d events per trigger), "
                               "%d tokens" % (args.stack, " -> ".join("FP16" if b == 16 else "INT%d" % b for b in ladder),
                                              per_trigger, T),
                   "order": "dependent" if dependent else "independent"},
        "speedup_over_first_rung": results["flexquant"] / results["fixed_%d" % ladder[0]],
        "events_fired": int(next_event), "events_total": n_events, "threshold_pple": thre,
        "first_switch_token": int(fired.min()) if fired.size else None,
        "last_switch_token": int(fired.max()) if fired.size else None,
        "average_weight_bits": avg_bits,
        "plan_status": {"gave_up": status[0], "flags": status[1]},
        "kl_order": {"first": [int(e) for e in order[:4]], "last": [int(e) for e in order[-4:]],
                     "kl_min": float(kl_host.min()), "kl_max": float(kl_host.max()),
                     "ascending": bool(np.all(np.diff(kl_host[order]) >= 0))}}
    for b in ladder:
        out["fixed_%s_tokens_per_s" % ("fp16" if b == 16 else "int%d" % b)] = results["fixed_%d" % b]
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="decode", choices=["decode", "prefill", "prefill-w8a8", "entropy", "flexquant", "quantize", "lm-head"],
                    help="decode = the headline decode stack (default); prefill / entropy = the "
                         "prefill-shaped GEMM slice and the batched entropy/KL on their own")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--stack", default="llama7b", choices=sorted(synth.STACKS))
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--bits", default="4,8", help="bit-widths drawn per layer per token")
    ap.add_argument("--shape", default=None, help="--workload prefill and prefill-w8a8: one shape NxK (weight rows x inputs) instead of both")
    ap.add_argument("--prefill-bits", default="4,8", help="--workload prefill: the bit-widths of the GEMMs of a step")
    ap.add_argument("--ladder", default="16,8,4", help="--workload flexquant: the formats a linear steps down through")
    ap.add_argument("--layers", type=int, default=None, help="truncate the stack (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB before the timed region "
                         "(calibrates HBM byte counters when profiling)")
    ap.add_argument("--verbose", action="store_true")
    ap.add_argument("--order", default="dependent", choices=["dependent", "independent"],
                    help="batch 1: the step's linears in the order a decoder must issue them (one launch of "
                         "the stage-ordered plan; default) or as one plan of independent entries")
    ap.add_argument("--w8a8-group", default="128", choices=["128", "row"],
                    help="--workload prefill-w8a8: the INT8 copy's scales, per group of 128 inputs (default) or one "
                         "per weight row (group = K)")
    ap.add_argument("--staged", action="store_true",
                    help="also time the dependent order as 4 separate plan launches per layer (HIP graph)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
                 "--gpus %d is not supported, run with --gpus 1" % args.gpus)

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    if args.workload == "prefill":
        return bench_prefill(args)
    if args.workload == "prefill-w8a8":
        return bench_prefill_w8a8(args)
    if args.workload == "entropy":
        return bench_entropy(args)
    if args.workload == "quantize":
        return bench_quantize(args)
    if args.workload == "lm-head":
        return bench_lm_head(args)
    if args.workload == "flexquant":
        return bench_flexquant(args)
    bit_choices = tuple(int(b) for b in args.bits.split(","))
    stack = Stack(args.stack, M=args.batch, bit_choices=bit_choices, layers=args.layers,
                  verbose=args.verbose)
    K_steps, W = args.steps, args.warmup
    fq = stack.fq
    # Order of the linears inside a step.  "dependent": the order a decoder must issue them in --
    # q/k/v, then o, then gate/up, then down, layer after layer, every group waiting for the one
    # before it (4 stages per decoder layer) -- as ONE launch of the stage-ordered plan.
    # "independent": all linears of the step as one plan of mutually independent entries (every
    # entry has its own seeded x in this workload, so both orders compute the same numbers); it is
    # the kernel-level figure for the weight stream.  Batches above 1 are served in the independent
    # order only.
    order = args.order if args.batch == 1 else "independent"
    if order == "dependent":
        stack.build_staged_plan()
        run_linears = stack.run_linears_one_launch_staged
        plan_of_step = stack.staged_plan
    else:
        run_linears = stack.run_linears
        plan_of_step = stack.plan
    if args.copy_mib > 0:
        src = torch.ones(args.copy_mib << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step(s):
        run_linears(s)
        stack.run_entropy(s)

    for s in range(W):
        step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(K_steps):
        step(W + s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    step_bytes = [stack.step_bytes(W + s) for s in range(K_steps)]
    total_bytes = float(sum(step_bytes))
    alg_bytes = total_bytes / K_steps

    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def time_launches(fn, n):
        """Mean duration of n back-to-back calls, from HIP events on the launch stream."""
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(n):
            fn(i)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # Dominant kernel of the timed step: the plan launch.
    lin_ms = time_launches(lambda i: run_linears(W + i), K_steps)
    ent_us = time_launches(lambda i: stack.run_entropy(W + i), K_steps) * 1e3

    def switching_cost(plan, mixed_ms):
        """The timed mixed patterns against what the same linears cost in the fixed-precision runs
        (each linear charged its share, by bytes, of the all-b run)."""
        n = len(stack.layers)
        fixed = {}
        for b in (4, 8):
            bd = torch.full((n,), b, dtype=torch.int32, device="cuda:0")
            time_launches(lambda i: plan.run(bd), 8)
            fixed[b] = time_launches(lambda i: plan.run(bd), K_steps)
        tot = {b: sum(weight_bytes(N, K, b) for (_, _, K, N) in stack.entries) for b in (4, 8)}
        pred = np.mean([sum(fixed[int(b)] * weight_bytes(N, K, int(b)) / tot[int(b)]
                            for (_, _, K, N), b in zip(stack.entries, stack.patterns[(W + s) % N_PATTERNS]))
                        for s in range(K_steps)])
        one = stack.bits_dev[W % N_PATTERNS]
        same_pattern = time_launches(lambda i: plan.run(one), K_steps)
        return {"all_w4_ms": fixed[4], "all_w8_ms": fixed[8], "mixed_ms": mixed_ms,
                "mixed_predicted_from_fixed_ms": float(pred), "overhead": mixed_ms / float(pred) - 1.0,
                "same_pattern_every_token_ms": same_pattern}

    switching = switching_cost(plan_of_step, lin_ms) if set(bit_choices) == {4, 8} else None

    # What this machine gives a kernel that only reads (same access pattern as the decode kernels).
    probe = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    probe.fill_(1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    time_launches(lambda i: fq.fq_stream_read(probe, probe.numel(), sink), 3)
    stream_gbps = probe.numel() / (time_launches(lambda i: fq.fq_stream_read(probe, probe.numel(), sink), 20) * 1e-3) / 1e9
    del probe

    traffic_key = (args.stack, args.batch, bit_choices)
    kernel_of = {"dependent": "decode_staged_kernel (one launch: %d stages)" % getattr(stack, "n_stages", 0),
                 "independent": "decode_m1_kernel (plan launch)" if args.batch == 1
                 else "decode_skinny_kernel (128-row tiles: the plan holds 3-bit copies)" if 3 in bit_choices
                 else "decode_stream_kernel"}

    def roofline(kernel, ms, traffic=None, traffic_source=None):
        achieved = alg_bytes / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "frac_of_measured_stream": achieved / stream_gbps,
                "traffic": traffic, "traffic_source": traffic_source,
                "avg_launch_ms": ms, "algorithmic_bytes_per_launch": alg_bytes}

    def measured_traffic(key=traffic_key):
        if args.layers is None and key in MEASURED_TRAFFIC_RATIO:
            return alg_bytes * MEASURED_TRAFFIC_RATIO[key], TRAFFIC_SOURCE[key]
        return None, None

    out = {
        "metric": "effective weight GB/s + decode tokens/s, mixed W4/W8 Llama-7B-shaped linears",
        "value": args.batch * K_steps / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K_steps, "warmup": W,
        "ms_per_step": elapsed / K_steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 x int%s -> f32" % "/int".join(str(b) for b in bit_choices if b != 16)
                 + (" (+ f16 x f16)" if 16 in bit_choices else ""),
        "data": "synthetic",
        "config": {"workload": "%s decode stack, batch %d, per-layer bits drawn from {%s} per token, "
                               "%d linears + entropy/KL over %d logits per step"
                               % (args.stack, args.batch, args.bits, len(stack.layers), VOCAB),
                   "order": order,
                   "launches_per_step": 2 if args.batch == 1 else 3,
                   "build_seconds": round(stack.build_seconds, 1)},
        "weight_GBps": total_bytes / elapsed / 1e9,
        "weight_GB_per_step": alg_bytes / 1e9,
        "entropy_kl_us": ent_us,
        "stream_read_GBps": stream_gbps,
    }
    if order == "dependent":
        out["roofline"] = roofline(kernel_of["dependent"], lin_ms, *measured_traffic(traffic_key + ("dependent",)))
        gave_up, flags = stack.staged_plan.status()
        out["staged_plan_status"] = {"gave_up": gave_up, "flags": flags}
        # beside it: the same linears as one plan of independent entries (the weight stream alone)
        for i in range(8):
            stack.run_linears(W + i)
        ind_ms = time_launches(lambda i: stack.run_linears(W + i), K_steps)
        traffic, source = measured_traffic()
        ind = {"ms_per_step": ind_ms + ent_us * 1e-3, "tokens_per_s": 1e3 / (ind_ms + ent_us * 1e-3),
               "roofline": roofline(kernel_of["independent"], ind_ms, traffic, source)}
        if set(bit_choices) == {4, 8}:
            ind["switching"] = switching_cost(stack.plan, ind_ms)
        out["independent_order"] = ind
        if args.staged:
            out.update(dependent_order_as_launches(stack, W, K_steps))
    else:
        traffic, source = measured_traffic()
        out["roofline"] = roofline(kernel_of["independent"], lin_ms, traffic, source)
        if args.staged:
            # batches above 1 have no stage-ordered launch: the dependent order is 4 plan launches per layer
            out.update(dependent_order_as_launches(stack, W, K_steps))
    if switching is not None:
        out["switching"] = switching
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(stack)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
