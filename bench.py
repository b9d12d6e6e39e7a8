#!/usr/bin/env python3
"""Benchmark of the melded FP8-LoRA linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path over one batch of synthetic input: melded forward,
melded backward (input gradient, adapter gradient, proxy-buffer step) and the row-wise proxy
update, at the LLaMA-7B attention-projection shape (T = n = m = 4096, r = 64, k = 32).
All inputs are resident in HBM before the timed region.  One JSON line is printed.

How the step is timed: at least W warm-up steps and never less than 0.3 s of them (the clocks need a
few dozen steps to settle after an idle period), then REPEATS blocks of exactly K steps, each block
bracketed by a device synchronisation; `ms_per_step` is the median block.  The step is issued call
by call through the C ABI; the same step captured once into a HIP graph and replayed is reported
beside it (`kernels.step_graph_ms`; on this chip the replay is not faster).
"""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

METRIC = "melded FP8 LoRA layer fwd+bwd tokens/sec and % FP8 MFMA peak, 7B shapes"
FP8_PEAK_TFLOPS = 5000.0       # MI355X dense FP8 MFMA, published
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
REPEATS = 5                    # timed blocks of K steps; the median is reported
WARMUP_FLOOR_S = 0.3
# Bytes that cross the L2 <-> fabric boundary per launch of the two product kernels at config 2:
# rocprofv3 --pmc FETCH_SIZE (scaled by the plain-copy calibration) + WRITE_SIZE runs of this command;
# the figures and the commands are in the committed summary named below.
TRAFFIC_SOURCE = "profiles/bench_config2_pmc_hbm_traffic_and_mfma.md"
TRAFFIC_BYTES = {"gemm_fwd_ride_kernel": 137.3e6, "gemm_dx_tail_kernel": 157.5e6}


def _events(fn, iters):
    """Average milliseconds per call of fn over `iters` back-to-back calls, by HIP events on
    the stream the kernels are launched on (torch's current stream)."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def _median_events(fn, iters, repeats=REPEATS):
    return statistics.median(_events(fn, iters) for _ in range(repeats))


def _wall_blocks(fn, steps, repeats=REPEATS):
    """`repeats` blocks of exactly `steps` calls, each bracketed by a device synchronisation; ms per call of every block."""
    out = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) * 1e3 / steps)
    return out


def _warm(fn, steps, floor_s=WARMUP_FLOOR_S):
    """At least `steps` calls and at least `floor_s` seconds of them."""
    done = 0
    t0 = time.perf_counter()
    while done < steps or time.perf_counter() - t0 < floor_s:
        for _ in range(10):
            fn()
        done += 10
        torch.cuda.synchronize()
    return done


def _capture(step):
    """The step as a HIP graph.  The library's calls only enqueue kernels on the caller's stream (no
    allocation, no memset, no synchronisation), so the whole step is capturable."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                 # code objects loaded, kernel attributes set, before the capture
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    return graph


def cpu_baseline(cfg, d, sample_tokens, reps):
    """The CPU oracle, as it stands, on the first `sample_tokens` tokens of the same workload
    taken as one batch: quantize, merged forward, backward and proxy update, `reps` times."""
    import oracle
    m, n, r, k = d["shape"].m, d["shape"].n, cfg.r, cfg.k
    x = d["x"][:sample_tokens].float().numpy()
    dy = d["dy"][:sample_tokens].float().numpy()
    wq, s_w, _ = oracle.quantize(d["w"].numpy(), oracle.E4M3)            # initialization: not timed
    aq, _, _ = oracle.quantize(d["a"].numpy(), oracle.E4M3, scale_in=s_w)
    wcat = np.concatenate([wq, aq])
    t0 = time.perf_counter()
    for _ in range(reps):
        f = oracle.layer_fwd(x, wcat, s_w, m, r)
        b = oracle.layer_bwd(dy, wcat, s_w, f["o_a"], f["amax_oa"], m, r,
                             delta_buf=np.zeros((m, r), np.float32), lr=cfg.lr)
        oracle.proxy_update(b["delta_buf"], wcat, m, r, k)
    dt = time.perf_counter() - t0
    return {"value": reps * sample_tokens / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {sample_tokens} of {cfg.T} tokens of the same workload ({m}x{n}) as one batch, "
                      f"fwd+bwd+update {reps} time(s) ({dt:.1f} s)"}


def bf16_lora_layer(T, n, m, r, iters):
    """Context only: an unquantized bf16 LoRA layer (separate adapter path) with library GEMMs."""
    dev = "cuda"
    g = torch.Generator(device=dev).manual_seed(1)
    x = torch.randn(T, n, device=dev, dtype=torch.bfloat16, generator=g)
    dy = torch.randn(T, m, device=dev, dtype=torch.bfloat16, generator=g)
    w = (torch.randn(m, n, device=dev, generator=g) * 0.02).to(torch.bfloat16)
    a = (torch.randn(r, n, device=dev, generator=g) / r).to(torch.bfloat16)
    b = torch.zeros(m, r, device=dev, dtype=torch.bfloat16)

    def step():
        xa = x @ a.t()
        y = x @ w.t() + xa @ b.t()
        dyb = dy @ b
        dx = dy @ w + dyb @ a
        db = dy.t() @ xa
        da = dyb.t() @ x
        return y, dx, db, da

    for _ in range(20):
        step()
    return _events(step, iters)


def library_fp8_gemm(T, n, m, iters):
    """Context only: the vendor library's FP8 GEMM (torch._scaled_mm, per-tensor scales, bf16 output)
    at the shape of the forward backbone product, on random E4M3 operands."""
    dev = "cuda"
    g = torch.Generator(device=dev).manual_seed(2)
    a = torch.randn(T, n, device=dev, generator=g).to(torch.float8_e4m3fn)
    b = torch.randn(m, n, device=dev, generator=g).to(torch.float8_e4m3fn)
    one = torch.ones((), device=dev)

    def run():
        return torch._scaled_mm(a, b.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16)

    for _ in range(20):
        run()
    return _events(run, iters)


def separate_path_fp8_lora_layer(fq, T, n, m, r, x, dy, w, a, iters):
    """Context only: a conventional FP8 LoRA layer with a separate adapter path, assembled from
    this library's own unfused kernels (quantizer, FP8 GEMM).  Per step it quantizes X, A, B, O_A,
    dY and dY.B and runs the backbone product plus four small-rank products; the two
    token-contracted adapter gradients use library bf16 GEMMs (which favours this path)."""
    dev = "cuda"
    u8, f32, bf16 = torch.uint8, torch.float32, torch.bfloat16
    ws = torch.empty(fq.workspace_bytes(T, n, m, r), dtype=u8, device=dev)
    wq = torch.empty(m, n, dtype=u8, device=dev); s_w = torch.zeros(1, device=dev)
    fq.quantize(w, fq.E4M3, wq, s_w, ws)
    b = (torch.randn(m, r, device=dev) * 0.01).to(bf16)
    xq = torch.empty(T, n, dtype=u8, device=dev); s_x = torch.zeros(1, device=dev)
    aq = torch.empty(r, n, dtype=u8, device=dev); s_a = torch.zeros(1, device=dev)
    bq = torch.empty(m, r, dtype=u8, device=dev); s_b = torch.zeros(1, device=dev)
    oa = torch.empty(T, r, dtype=bf16, device=dev); oaq = torch.empty(T, r, dtype=u8, device=dev); s_oa = torch.zeros(1, device=dev)
    y0 = torch.empty(T, m, dtype=bf16, device=dev); y1 = torch.empty(T, m, dtype=bf16, device=dev)
    dyq = torch.empty(T, m, dtype=u8, device=dev); s_dy = torch.zeros(1, device=dev)
    dx0 = torch.empty(T, n, dtype=bf16, device=dev); dx1 = torch.empty(T, n, dtype=bf16, device=dev)
    g = torch.empty(T, r, dtype=bf16, device=dev); gq = torch.empty(T, r, dtype=u8, device=dev); s_g = torch.zeros(1, device=dev)
    a_bf = a.to(bf16)

    def step():
        fq.quantize(x, fq.E4M3, xq, s_x, ws)
        fq.quantize(a_bf, fq.E4M3, aq, s_a, ws)
        fq.quantize(b, fq.E4M3, bq, s_b, ws)
        fq.fp8_gemm(xq, fq.E4M3, wq, False, s_x, s_w, y0)
        fq.fp8_gemm(xq, fq.E4M3, aq, False, s_x, s_a, oa)
        fq.quantize(oa, fq.E4M3, oaq, s_oa, ws)
        fq.fp8_gemm(oaq, fq.E4M3, bq, False, s_oa, s_b, y1)
        y = y0 + y1
        fq.quantize(dy, fq.E5M2, dyq, s_dy, ws)
        fq.fp8_gemm(dyq, fq.E5M2, wq, True, s_dy, s_w, dx0)
        fq.fp8_gemm(dyq, fq.E5M2, bq, True, s_dy, s_b, g)
        fq.quantize(g, fq.E5M2, gq, s_g, ws)
        fq.fp8_gemm(gq, fq.E5M2, aq, True, s_g, s_a, dx1)
        dx = dx0 + dx1
        db = dy.t() @ oa
        da = g.t() @ x
        return y, dx, db, da

    for _ in range(20):
        step()
    return _events(step, iters)


def _layer_flops(T, n, m, r):
    return 2.0 * T * n * (m + r) + 2.0 * T * m * n + 2.0 * T * m * r


def run_stack(fq, cfg, args):
    """Configs with several layers: every projection of the config as its own melded layer (own
    weights, buffer and saved O_A; per-step activations shared between layers of one shape, which
    run one after the other).  A step is forward over all layers, backward over all layers in
    reverse; the proxy update of every layer follows each `accumulate_steps`-th step."""
    T, r, k = cfg.T, cfg.r, cfg.k
    layers, inputs = [], []
    for li, shape in enumerate(cfg.layers):
        d = workloads.config_layer_inputs(cfg.cfg, li)
        w, a = d["w"].cuda(), d["a"].cuda()
        first = None
        for _ in range(shape.count):
            layer = fq.MeldedLinear(T, shape.n, shape.m, r, k, out_dtype=torch.bfloat16, share_transients_with=first)
            layer.init_weights(w, a)
            first = first or layer
            layers.append(layer)
            inputs.append(li)
        del w, a
    xs = [workloads.config_layer_inputs(cfg.cfg, li)["x"].cuda() for li in range(len(cfg.layers))]
    dys = [workloads.config_layer_inputs(cfg.cfg, li)["dy"].cuda() for li in range(len(cfg.layers))]
    acc = cfg.accumulate_steps

    def train_step(i):
        for layer, li in zip(layers, inputs):
            layer.forward(xs[li])
        for layer, li in zip(reversed(layers), reversed(inputs)):
            layer.backward(dys[li], lr=cfg.lr)
        if (i + 1) % acc == 0:
            for layer in layers:
                layer.update(reuse_scores=True)

    def cycle():                                   # one whole accumulation cycle
        for i in range(acc):
            train_step(i)

    # whole accumulation cycles; at most about 10 s of timed work and 2 s of warm-up
    cycle()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    cycle()
    torch.cuda.synchronize()
    est = (time.perf_counter() - t0) / acc
    warm = max(min(args.warmup, int(2.0 / est)), acc) // acc
    cycles = max(min(args.steps, int(10.0 / est) // REPEATS), acc) // acc
    _warm(cycle, warm)
    blocks = [b / acc for b in _wall_blocks(cycle, cycles)]
    ms_per_step = statistics.median(blocks)
    flops = sum(s.count * _layer_flops(T, s.n, s.m, r) for s in cfg.layers)
    n_layers = len(layers)
    desc = ", ".join(f"{s.count}x {s.m}x{s.n}" for s in cfg.layers)
    out = {
        "metric": METRIC, "value": T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": cycles * acc, "warmup": warm * acc, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8 (E4M3 weights/activations, E5M2 gradients), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.cfg} ({cfg.name}): T={T}, {n_layers} layers ({desc}), r={r}, k={k}; "
                               f"fwd + bwd over all layers per step, proxy update of every layer each "
                               f"{acc} step(s) (its time is spread over them)",
                   "launch": "call by call", "repeats": REPEATS, "ms_per_step_blocks": blocks},
        "roofline": {"bound": "mfma", "kernel": "all FP8 products of the step (whole-step time, not a kernel time)",
                     "achieved": flops / (ms_per_step * 1e-3) / 1e12, "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / (ms_per_step * 1e-3) / 1e12 / FP8_PEAK_TFLOPS, "traffic": None},
        "kernels": {"gemm_flops_per_step": flops, "layers": n_layers},
    }
    print(json.dumps(out))


def rank_sweep(fq, cfg, args):
    """Context table: fwd+bwd time of the melded layer, of the separate-path FP8 LoRA layer and of
    the bf16 LoRA layer at the headline shape for every adapter rank the library takes (the
    paper's preliminary analysis and its rank-efficiency table compare FP8 and FP16 adapters over
    ranks on its own hardware).  Prints one JSON line."""
    d = workloads.config_layer_inputs(cfg.cfg, 0)
    m, n, T = d["shape"].m, d["shape"].n, cfg.T
    x, dy, w = d["x"].cuda(), d["dy"].cuda(), d["w"].cuda()
    it = max(10, args.steps)
    rows = []
    for r in (16, 32, 64, 128, 256):
        a = (torch.randn(r, n, generator=torch.Generator().manual_seed(r)) / r).cuda()
        layer = fq.MeldedLinear(T, n, m, r, cfg.k, out_dtype=torch.bfloat16)
        layer.init_weights(w, a)
        for _ in range(3):
            layer.forward(x); layer.backward(dy, lr=cfg.lr)
        ms_melded = _events(lambda: (layer.forward(x), layer.backward(dy, lr=cfg.lr)), it)
        ms_sep = separate_path_fp8_lora_layer(fq, T, n, m, r, x, dy, w, a, it)
        ms_bf16 = bf16_lora_layer(T, n, m, r, it)
        rows.append({"r": r, "melded_fwd_bwd_ms": ms_melded, "separate_path_fp8_ms": ms_sep, "bf16_lora_ms": ms_bf16,
                     "melded_vs_separate_fp8": ms_sep / ms_melded, "melded_vs_bf16": ms_bf16 / ms_melded,
                     "separate_fp8_vs_bf16": ms_bf16 / ms_sep})
        del layer
    print(json.dumps({"rank_sweep": rows, "workload": f"T={T}, n={n}, m={m} (config {cfg.cfg} shape), fwd+bwd per layer",
                      "data": "synthetic"}))


def decoder_block(fq, args):
    """Context: one LLaMA-13B-shaped decoder block (d = 5120, 40 heads, MLP 13824, 8 x 1024 tokens)
    forward + backward with real data dependence between its seven projections: melded layers
    against bf16 LoRA layers (frozen W, trainable A and B) in the same block.  Prints one JSON line."""
    from paper_2510_24061_amd.nn import LlamaBlock, MeldedLoRALinear
    d_model, heads, d_mlp, r, k, batch, seq = 5120, 40, 13824, 64, 64, 8, 1024
    g = torch.Generator(device="cuda").manual_seed(13)

    def melded(i, o):
        lin = MeldedLoRALinear(i, o, r, k, sgd_lr=2e-4)
        lin.load_weights(torch.randn(o, i, device="cuda", generator=g) * 0.02,
                         torch.randn(r, i, device="cuda", generator=g) / r)
        return lin

    class LoRALinear(torch.nn.Module):
        def __init__(self, i, o):
            super().__init__()
            self.w = torch.nn.Parameter((torch.randn(o, i, device="cuda", generator=g) * 0.02).to(torch.bfloat16),
                                        requires_grad=False)
            self.a = torch.nn.Parameter((torch.randn(r, i, device="cuda", generator=g) / r).to(torch.bfloat16))
            self.b = torch.nn.Parameter(torch.zeros(o, r, device="cuda", dtype=torch.bfloat16))

        def forward(self, x):
            return x @ self.w.t() + (x @ self.a.t()) @ self.b.t()

    x = torch.randn(batch, seq, d_model, device="cuda", generator=g).to(torch.bfloat16)
    out = {}
    for name, make in (("melded_fp8", melded), ("bf16_lora", LoRALinear)):
        block = LlamaBlock(d_model, heads, d_mlp, make)
        xin = x.clone().requires_grad_(True)

        def step():
            y = block(xin)
            y.backward(y.detach())                          # any gradient of the right shape

        for _ in range(5):
            step()
        out[name + "_ms"] = _events(step, max(10, min(args.steps, 50)))
        del block
    out["speedup"] = out["bf16_lora_ms"] / out["melded_fp8_ms"]
    out["backbone_gemm_flops"] = 2 * 2.0 * batch * seq * (4 * d_model * d_model + 3 * d_model * d_mlp)   # fwd + dX
    out["workload"] = (f"decoder block d={d_model}, heads={heads}, mlp={d_mlp}, tokens={batch}x{seq}, r={r}: "
                       "fwd+bwd, PyTorch RMSNorm / causal attention / SwiGLU between the projections")
    print(json.dumps({"decoder_block": out, "data": "synthetic"}))


def _product_launches(fq, layer, x, dy, cfg):
    """The two product launches of a step, each issued alone through falqon_fp8_gemm exactly as
    falqon_melded_fwd / falqon_melded_bwd issue it (backbone product whose workgroups also form the
    adapter's product), on the step's own operands.  Returns (forward fn, backward fn)."""
    T, n, m, r = layer.T, layer.n, layer.m, layer.r
    layer.forward(x)
    layer.backward(dy, lr=cfg.lr)
    oa_codes = torch.empty(T, r, dtype=torch.uint8, device="cuda")
    s_oa = (448.0 / torch.clamp(layer.amax_oa, min=1e-12)).float()
    s_tmp = torch.zeros(1, device="cuda")
    fq.quantize(layer.o_a, fq.E4M3, oa_codes, s_tmp, layer.ws, scale_in=s_oa)
    side_ws = torch.empty_like(layer.ws)
    y_tmp, dx_tmp = torch.empty_like(layer.y), torch.empty_like(layer.dx)
    wq_b, wq_a = layer.wq[:m], layer.wq[m:]

    def fwd():
        fq.fp8_gemm(layer.xq, fq.E4M3, wq_b, False, layer.s_x, layer.s_w, y_tmp, side=wq_a, side_ws=side_ws)

    def bwd():
        fq.fp8_gemm(layer.dyq, fq.E5M2, wq_b, True, layer.s_dy, layer.s_w, dx_tmp, side=oa_codes, side_ws=side_ws)

    fwd(); bwd()                       # raises where the melded calls do not use these launches (small or odd shapes)
    torch.cuda.synchronize()
    assert torch.equal(y_tmp, layer.y) and torch.equal(dx_tmp, layer.dx)     # the same launches, the same bytes
    return fwd, bwd


def layer_summary(fq, cfg_id, layer_index, steps, cpu_tokens, with_cpu):
    """One layer of another configuration, time-capped: ms per fwd + bwd + update (median of blocks),
    its two product launches alone, and a CPU-oracle sample."""
    cfg = workloads.CONFIGS[cfg_id]
    d = workloads.config_layer_inputs(cfg_id, layer_index)
    m, n, r, k, T = d["shape"].m, d["shape"].n, cfg.r, cfg.k, cfg.T
    layer = fq.MeldedLinear(T, n, m, r, k, out_dtype=torch.bfloat16)
    layer.init_weights(d["w"].cuda(), d["a"].cuda())
    x, dy = d["x"].cuda(), d["dy"].cuda()

    def step():
        layer.forward(x)
        layer.backward(dy, lr=cfg.lr)
        layer.update(reuse_scores=True)

    _warm(step, 50)
    blocks = _wall_blocks(step, steps)
    ms = statistics.median(blocks)
    fwd, bwd = _product_launches(fq, layer, x, dy, cfg)
    ms_f, ms_b = _median_events(fwd, max(100, steps // 4)), _median_events(bwd, max(100, steps // 4))
    fl_f, fl_b = 2.0 * T * n * (m + r), 2.0 * T * m * n + 2.0 * T * m * r
    out = {"workload": f"config {cfg_id} layer {layer_index} ({d['shape'].name}): T={T}, n={n}, m={m}, r={r}, k={k}; "
                       "fwd + bwd + proxy update per step",
           "ms_per_step": ms, "ms_per_step_blocks": blocks, "tokens_per_s": T / (ms * 1e-3),
           "products_flops": fl_f + fl_b,
           "whole_step": {"TFLOP/s": (fl_f + fl_b) / (ms * 1e-3) / 1e12, "frac_fp8_peak": (fl_f + fl_b) / (ms * 1e-3) / 1e12 / FP8_PEAK_TFLOPS},
           "product_launches": {
               "forward_ms": ms_f, "backward_ms": ms_b,
               "TFLOP/s": (fl_f + fl_b) / ((ms_f + ms_b) * 1e-3) / 1e12,
               "frac_fp8_peak": (fl_f + fl_b) / ((ms_f + ms_b) * 1e-3) / 1e12 / FP8_PEAK_TFLOPS}}
    del layer, x, dy
    torch.cuda.empty_cache()
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, d, min(cpu_tokens, T), 1)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2, help="workload (2 = the headline LLaMA-7B attention projection; 3-5 run all their layers as a stack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the bf16 LoRA and separate-path FP8 LoRA comparison layers and the other configurations' "
                         "layers (profiling runs: their launches of the same kernels at other sizes would blur the "
                         "per-kernel statistics)")
    ap.add_argument("--decoder-block", action="store_true",
                    help="print the decoder-block context measurement instead of the benchmark line")
    ap.add_argument("--rank-sweep", action="store_true",
                    help="print the rank-sweep context table instead of the benchmark line")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    ap.add_argument("--cpu-reps", type=int, default=4)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)

    import paper_2510_24061_amd as fq

    cfg = workloads.CONFIGS[args.config]
    if args.rank_sweep:
        rank_sweep(fq, cfg, args)
        return
    if args.decoder_block:
        decoder_block(fq, args)
        return
    if sum(s.count for s in cfg.layers) > 1:
        run_stack(fq, cfg, args)
        return
    d = workloads.config_layer_inputs(args.config, 0)
    m, n, r, k, T = d["shape"].m, d["shape"].n, cfg.r, cfg.k, cfg.T
    layer = fq.MeldedLinear(T, n, m, r, k, out_dtype=torch.bfloat16)
    layer.init_weights(d["w"].cuda(), d["a"].cuda())
    x, dy = d["x"].cuda(), d["dy"].cuda()
    torch.cuda.synchronize()

    def step():
        layer.forward(x)
        layer.backward(dy, lr=cfg.lr)
        layer.update(reuse_scores=True)

    # ---- the timed region: median of REPEATS blocks of K steps ----
    warm_done = _warm(step, args.warmup)
    blocks = _wall_blocks(step, args.steps)
    ms_per_step = statistics.median(blocks)
    # the same step captured into a HIP graph and replayed
    graph = _capture(step)
    _warm(graph.replay, 20, 0.05)
    ms_graph = statistics.median(_wall_blocks(graph.replay, args.steps))

    # ---- per-call and per-kernel timing (HIP events on the launch stream) -------------------
    it = max(500, args.steps)                      # launches per event-timed run, whatever K the step loop uses
    ms_fwd = _median_events(lambda: layer.forward(x), it)
    ms_bwd = _median_events(lambda: layer.backward(dy, lr=cfg.lr), it)
    # without clearing, so that the buffer keeps its content over the repeated calls (a cleared buffer ends up all
    # zero, a degenerate case: every row ties and the first k rows, all neighbours, are selected)
    ms_upd = _median_events(lambda: layer.update(clear_selected=False), it)
    # the two product launches of the step, each alone, exactly as the melded calls issue them
    fwd_launch, bwd_launch = _product_launches(fq, layer, x, dy, cfg)
    ms_prod_fwd = _median_events(fwd_launch, it)
    ms_prod_bwd = _median_events(bwd_launch, it)
    # the plain backbone products (no side job), for comparison
    y_tmp = torch.empty(T, m, dtype=torch.bfloat16, device="cuda")
    ms_gemm_fwd = _median_events(lambda: fq.fp8_gemm(layer.xq, fq.E4M3, layer.wq[:m], False, layer.s_x, layer.s_w, y_tmp), it)
    ms_gemm_dx = _median_events(lambda: fq.fp8_gemm(layer.dyq, fq.E5M2, layer.wq[:m], True, layer.s_dy, layer.s_w, layer.dx), it)
    ms_gemm_const = None
    if not args.no_context:
        # the plain product on constant operands (every code = 1.0): identical instruction stream and memory traffic,
        # but almost no switching in the multipliers, so the chip holds its full clock - the rate the kernel's
        # schedule reaches when the power management does not intervene
        ones_x, ones_w = torch.full_like(layer.xq, 0x38), torch.full_like(layer.wq[:m], 0x38)
        ms_gemm_const = _median_events(lambda: fq.fp8_gemm(ones_x, fq.E4M3, ones_w, False, layer.s_x, layer.s_w, y_tmp), it)
        del ones_x, ones_w
    # optimizer variant of the buffer step: bwd without the SGD step, global-norm term, AdamW into the buffer
    sum_sq = torch.zeros(1, dtype=torch.float64, device="cuda")
    layer.adamw_step(1, sum_sq)                       # allocates the moments
    ms_sqnorm = _events(lambda: fq.grad_sqnorm(layer.d_b, sum_sq, layer.ws), it)
    ms_adamw = _events(lambda: layer.adamw_step(2, sum_sq), it)
    # variant of the adapter gradient with O_A kept in bf16 (its two launches)
    db_tmp = torch.empty(m, r, device="cuda")
    ms_db_wide = _events(lambda: fq.db_bf16(layer.dyq, layer.s_dy, layer.o_a, db_tmp, None, 0.0, layer.ws), it)
    del db_tmp
    # variant that also forms the gradient of the adapter factor A (the paper's "+ Update matrix A" ablation row):
    # two more products per layer step, on a random B^ cast to E4M3
    bt = torch.randn(r, m, device="cuda", generator=torch.Generator(device="cuda").manual_seed(5)) * 0.05
    btq = torch.empty(r, m, dtype=torch.uint8, device="cuda"); s_b = torch.zeros(1, device="cuda")
    fq.quantize(bt, fq.E4M3, btq, s_b, layer.ws)
    g_tmp = torch.empty(T, r, dtype=torch.bfloat16, device="cuda"); amax_g = torch.zeros(1, device="cuda")
    dat_tmp = torch.empty(n, r, device="cuda")
    ws_da = torch.empty(fq.workspace_bytes(T, m, n, r), dtype=torch.uint8, device="cuda")
    ms_da = _median_events(lambda: fq.da(layer.dyq, layer.s_dy, btq, s_b, layer.xq, layer.s_x, g_tmp, amax_g, dat_tmp, ws_da), it)
    del bt, btq, g_tmp, dat_tmp, ws_da
    layer.delta_buf.zero_()
    s_tmp = torch.zeros(1, device="cuda")
    ms_quant = _median_events(lambda: fq.quantize(x, fq.E4M3, layer.xq, s_tmp, layer.ws), it)
    del y_tmp

    # one plain device-to-device copy of known size: the reference that scales the FETCH_SIZE /
    # WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    calib = torch.empty_like(x)
    calib.copy_(x)
    torch.cuda.synchronize()
    del calib

    flops_fwd = 2.0 * T * n * (m + r)              # backbone product + adapter columns: one launch
    flops_bwd = 2.0 * T * m * n + 2.0 * T * m * r  # input gradient + adapter gradient: one launch
    flops_plain = 2.0 * T * n * m
    quant_bytes = 3.0 * T * n                      # read bf16 once (second read is cache-served), write FP8
    upd_bytes = 4.0 * m * r + 2.0 * k * n + r * n + 8.0 * k * r   # scores + selected rows in/out + adapter rows + buffer rows
    # The dominant kernel of the step: the forward product launch (the backward one takes about as long).
    dominant_fwd = ms_prod_fwd >= ms_prod_bwd
    dom_ms, dom_flops = (ms_prod_fwd, flops_fwd) if dominant_fwd else (ms_prod_bwd, flops_bwd)
    traffic = TRAFFIC_BYTES["gemm_fwd_ride_kernel" if dominant_fwd else "gemm_dx_tail_kernel"]
    roofline = {
        "bound": "mfma",
        "kernel": ("gemm_fwd_ride_kernel (the product launch of falqon_melded_fwd: 256 tiles of 256x256 of X~ W~^T, the "
                   "blocks of O_A formed inside the tiles' own K-steps)") if dominant_fwd else
                  ("gemm_dx_tail_kernel (the product launch of falqon_melded_bwd: 256 tiles of 256x256 of dY~ W~, each "
                   "preceded by its share of dB)"),
        "achieved": dom_flops / (dom_ms * 1e-3) / 1e12, "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": dom_flops / (dom_ms * 1e-3) / 1e12 / FP8_PEAK_TFLOPS,
        "traffic": traffic, "traffic_source": TRAFFIC_SOURCE + " (rocprofv3 --pmc FETCH_SIZE x calibration + WRITE_SIZE of "
                                              "this command: bytes per launch at the L2-fabric boundary, a recorded figure)",
        "flops_per_launch": dom_flops, "avg_launch_ms": dom_ms,
        "how": "the launch issued alone through falqon_fp8_gemm(side=...) with the step's own operands, back to back, "
               "HIP events on the launch stream, median of %d runs" % REPEATS,
    }
    if ms_gemm_const is not None:
        roofline["plain_product_constant_operands"] = {
            "ms": ms_gemm_const, "TFLOP/s": flops_plain / (ms_gemm_const * 1e-3) / 1e12,
            "frac": flops_plain / (ms_gemm_const * 1e-3) / 1e12 / FP8_PEAK_TFLOPS,
            "note": "the plain backbone product with all codes = 1.0 (same kernel, grid and traffic): the clock stays at its "
                    "nominal value; the gap to kernels.gemm_fwd_plain is the clock the chip grants for the workload's bits"}
    tf = lambda fl, ms: fl / (ms * 1e-3) / 1e12
    kernels = {
        "step_eager_ms": ms_per_step, "step_graph_ms": ms_graph,
        "product_launch_fwd": {"ms": ms_prod_fwd, "flops": flops_fwd, "TFLOP/s": tf(flops_fwd, ms_prod_fwd),
                               "frac_fp8_peak": tf(flops_fwd, ms_prod_fwd) / FP8_PEAK_TFLOPS},
        "product_launch_bwd": {"ms": ms_prod_bwd, "flops": flops_bwd, "TFLOP/s": tf(flops_bwd, ms_prod_bwd),
                               "frac_fp8_peak": tf(flops_bwd, ms_prod_bwd) / FP8_PEAK_TFLOPS},
        "product_launches": {"ms": ms_prod_fwd + ms_prod_bwd, "flops": flops_fwd + flops_bwd,
                             "TFLOP/s": tf(flops_fwd + flops_bwd, ms_prod_fwd + ms_prod_bwd),
                             "frac_fp8_peak": tf(flops_fwd + flops_bwd, ms_prod_fwd + ms_prod_bwd) / FP8_PEAK_TFLOPS,
                             "note": "all three products of a step (forward with adapter columns, dX, dB) over their two launches"},
        "gemm_fwd_plain": {"ms": ms_gemm_fwd, "TFLOP/s": tf(flops_plain, ms_gemm_fwd), "frac_fp8_peak": tf(flops_plain, ms_gemm_fwd) / FP8_PEAK_TFLOPS,
                           "note": "backbone product alone, no side job (isolated launch, not part of the step)"},
        "gemm_dx_plain": {"ms": ms_gemm_dx, "TFLOP/s": tf(flops_plain, ms_gemm_dx), "frac_fp8_peak": tf(flops_plain, ms_gemm_dx) / FP8_PEAK_TFLOPS},
        "quantize_x": {"ms": ms_quant, "GB/s": quant_bytes / (ms_quant * 1e-3) / 1e9,
                       "frac_hbm_peak": quant_bytes / (ms_quant * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "proxy_update": {"ms": ms_upd, "GB/s": upd_bytes / (ms_upd * 1e-3) / 1e9,
                         "frac_hbm_peak": upd_bytes / (ms_upd * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "note": "dependent launches over 1.6 MB: latency bound"},
        "adamw_buffer_step": {"grad_sqnorm_ms": ms_sqnorm, "adamw_delta_ms": ms_adamw,
                              "bytes": 28.0 * m * r, "GB/s": 28.0 * m * r / (ms_adamw * 1e-3) / 1e9,
                              "note": "optional replacement of the SGD buffer step inside melded_bwd; not in the timed step"},
        "db_bf16_variant": {"ms": ms_db_wide, "flops": 2.0 * T * m * r,
                            "note": "dB = dy~^T O_A with O_A kept in bf16 (bf16 matrix cores), partial pass + ordered sum as "
                                    "two launches of their own; not in the timed step"},
        "a_update_variant": {"da_ms": ms_da, "flops": 4.0 * T * m * r if n == m else 2.0 * T * r * (m + n),
                             "step_with_da_ms": ms_per_step + ms_da, "slowdown": (ms_per_step + ms_da) / ms_per_step,
                             "note": "falqon_da, the gradient of the adapter factor A (dL/dA = B^T dL/dO x^T) as two small "
                                     "products; not in the timed step.  Paper, whole model on its GPU: 1.94 s against 1.80 s "
                                     "per step (7B), 3.89 against 3.26 (13B) - context only"},
        "calls": {"melded_fwd_ms": ms_fwd, "melded_bwd_ms": ms_bwd, "proxy_update_ms": ms_upd},
    }

    ms_fwd_bwd = ms_fwd + ms_bwd
    context = {"melded_fwd_bwd_ms": ms_fwd_bwd, "melded_fwd_bwd_update_ms": ms_per_step,
               "paper": "about 3x over prior quantized-LoRA methods, 1.22x over separate-path FP8, on one RTX 4090"}
    if not args.no_context:
        ms_bf16 = bf16_lora_layer(T, n, m, r, max(5, args.steps // 2))
        ms_sep = separate_path_fp8_lora_layer(fq, T, n, m, r, x, dy, d["w"].cuda(), d["a"].cuda(),
                                              max(5, args.steps // 2))
        try:
            context["library_fp8_gemm_ms"] = library_fp8_gemm(T, n, m, max(5, args.steps // 2))
        except Exception as exc:  # the library path is context only; its absence must not fail the benchmark
            context["library_fp8_gemm_ms"] = None
            context["library_fp8_gemm_error"] = repr(exc)[:200]
        context.update({"bf16_lora_layer_ms": ms_bf16, "separate_path_fp8_lora_layer_ms": ms_sep,
                        "speedup_vs_separate_path_fp8": ms_sep / ms_fwd_bwd,
                        "speedup_vs_bf16_lora": ms_bf16 / ms_fwd_bwd})

    out = {
        "metric": METRIC, "value": T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8 (E4M3 weights/activations, E5M2 gradients), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.cfg} ({cfg.name}): T={T}, n={n}, m={m}, r={r}, k={k}; "
                               "fwd + bwd + proxy update per step",
                   "launch": "call by call through the C ABI", "repeats": REPEATS,
                   "warmup_steps_done": warm_done,      # W, or as many steps as the warm-up floor (seconds) takes
                   "ms_per_step_blocks": blocks},
        "roofline": roofline, "kernels": kernels, "context": context,
    }
    del layer, graph
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, d, min(args.cpu_sample_tokens, T), args.cpu_reps)
        if args.config == 2:
            c1 = workloads.CONFIGS[1]
            out["cpu_baseline_config1"] = cpu_baseline(c1, workloads.config_layer_inputs(1), c1.T, 20)
    if not args.no_context and args.config == 2:
        # the two MLP projections of the same model (config 3) and of the 13B block (config 4), time-capped
        sub_steps = max(20, min(200, args.steps))
        out["configs"] = [layer_summary(fq, 3, li, sub_steps, 1024, not args.no_cpu_baseline) for li in (0, 1)]
        out["configs"] += [layer_summary(fq, 4, li, max(20, sub_steps // 2), 512, not args.no_cpu_baseline) for li in (1, 2)]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
