#!/usr/bin/env python3
"""Benchmark of the melded FP8-LoRA linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path over one batch of synthetic input: melded forward,
melded backward (input gradient, adapter gradient, proxy-buffer step) and the row-wise proxy
update, at the LLaMA-7B attention-projection shape (T = n = m = 4096, r = 64, k = 32).
All inputs are resident in HBM before the timed region.  One JSON line is printed.
The defaults (100 warm-up steps, 1000 timed steps, 0.2 s of GPU time) are long enough for the
clocks to settle: the first few dozen steps after an idle period run about 10 % slower.
"""
import argparse
import json
import os
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
# HBM bytes per launch of the forward GEMM kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# runs of this command (profiles/bench_config2_pmc_hbm_traffic_and_mfma.md).
GEMM_FWD_TRAFFIC_BYTES = 134.7e6   # 101.1 MB fetched (FETCH_SIZE x 1.998) + 33.6 MB written


def _time_region(fn, iters):
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
            "sample": f"first {sample_tokens} of {cfg.T} tokens of the same workload as one batch, "
                      f"fwd+bwd+update {reps} times ({dt:.1f} s)"}


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
    return _time_region(step, iters)


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
    return _time_region(run, iters)


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
    return _time_region(step, iters)


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
                layer.update()

    # whole accumulation cycles; at most about 10 s of timed work and 2 s of warm-up
    for i in range(acc):
        train_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(acc):
        train_step(i)
    torch.cuda.synchronize()
    est = (time.perf_counter() - t0) / acc
    warm = max(min(args.warmup, int(2.0 / est)), acc) // acc * acc
    steps = max(min(args.steps, int(10.0 / est)), acc) // acc * acc
    for i in range(warm):
        train_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        train_step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    flops = sum(s.count * (2.0 * T * s.n * (s.m + r) + 2.0 * T * s.m * s.n + 2.0 * T * s.m * r) for s in cfg.layers)
    n_layers = len(layers)
    desc = ", ".join(f"{s.count}x {s.m}x{s.n}" for s in cfg.layers)
    out = {
        "metric": METRIC, "value": T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warm, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8 (E4M3 weights/activations, E5M2 gradients), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.cfg} ({cfg.name}): T={T}, {n_layers} layers ({desc}), r={r}, k={k}; "
                               f"fwd + bwd over all layers per step, proxy update of every layer each "
                               f"{acc} step(s) (its time is spread over them)"},
        "roofline": {"bound": "mfma", "kernel": "all FP8 GEMMs of the step (whole-step time, not a kernel time)",
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
        ms_melded = _time_region(lambda: (layer.forward(x), layer.backward(dy, lr=cfg.lr)), it)
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
        out[name + "_ms"] = _time_region(step, max(10, min(args.steps, 50)))
        del block
    out["speedup"] = out["bf16_lora_ms"] / out["melded_fp8_ms"]
    out["backbone_gemm_flops"] = 2 * 2.0 * batch * seq * (4 * d_model * d_model + 3 * d_model * d_mlp)   # fwd + dX
    out["workload"] = (f"decoder block d={d_model}, heads={heads}, mlp={d_mlp}, tokens={batch}x{seq}, r={r}: "
                       "fwd+bwd, PyTorch RMSNorm / causal attention / SwiGLU between the projections")
    print(json.dumps({"decoder_block": out, "data": "synthetic"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2, help="workload (2 = the headline LLaMA-7B attention projection; 3-5 run all their layers as a stack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the bf16 LoRA and separate-path FP8 LoRA comparison layers (profiling runs: their "
                         "launches of the same GEMM kernel at other sizes would blur its per-kernel statistics)")
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
        layer.update()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- per-call and per-kernel timing (HIP events on the launch stream) -------------------
    it = max(10, args.steps)
    ms_fwd = _time_region(lambda: layer.forward(x), it)
    ms_bwd = _time_region(lambda: layer.backward(dy, lr=cfg.lr), it)
    ms_upd = _time_region(lambda: layer.update(), it)
    # the forward backbone product launched on its own (inside falqon_melded_fwd the same tile code shares
    # its launch with the adapter's split-K tiles)
    y_tmp = torch.empty(T, m, dtype=torch.bfloat16, device="cuda")
    ms_gemm_fwd = _time_region(lambda: fq.fp8_gemm(layer.xq, fq.E4M3, layer.wq[:m], False, layer.s_x, layer.s_w, y_tmp), it)
    ms_gemm_dx = _time_region(lambda: fq.fp8_gemm(layer.dyq, fq.E5M2, layer.wq[:m], True, layer.s_dy, layer.s_w,
                                                  layer.dx), it)
    ms_gemm_const = ms_probe = tflops_probe = None
    if not args.no_context:
        # the same launch on constant operands (every code = 1.0): identical instruction stream and memory traffic,
        # but almost no switching in the multipliers, so the chip holds its full clock - the rate the kernel's
        # schedule reaches when the power management does not intervene
        ones_x, ones_w = torch.full_like(layer.xq, 0x38), torch.full_like(layer.wq[:m], 0x38)
        ms_gemm_const = _time_region(lambda: fq.fp8_gemm(ones_x, fq.E4M3, ones_w, False, layer.s_x, layer.s_w, y_tmp), it)
        del ones_x, ones_w
        # the same matrix-core work as one backbone product (256 workgroups x 4 waves x 64 rounds x 16 instructions
        # of 32x32x64) from registers only, on the workload's own codes: the rate the chip sustains with no memory
        # traffic at all for these operand bits (its clock under matrix-core load falls as the bits toggle more)
        sink = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
        probe_rounds = n // 64
        ms_probe = _time_region(lambda: fq.mfma_probe(layer.xq, layer.wq, 256, probe_rounds, sink), it)
        tflops_probe = 256 * 4 * probe_rounds * 16 * 2.0 * 32 * 32 * 64 / (ms_probe * 1e-3) / 1e12
        del sink
    # optimizer variant of the buffer step: bwd without the SGD step, global-norm term, AdamW into the buffer
    sum_sq = torch.zeros(1, dtype=torch.float64, device="cuda")
    layer.adamw_step(1, sum_sq)                       # allocates the moments
    ms_sqnorm = _time_region(lambda: fq.grad_sqnorm(layer.d_b, sum_sq, layer.ws), it)
    ms_adamw = _time_region(lambda: layer.adamw_step(2, sum_sq), it)
    # variant of the adapter gradient with O_A kept in bf16 (its two launches, outside the paired launch)
    db_tmp = torch.empty(m, r, device="cuda")
    ms_db_wide = _time_region(lambda: fq.db_bf16(layer.dyq, layer.s_dy, layer.o_a, db_tmp, None, 0.0, layer.ws), it)
    del db_tmp
    layer.delta_buf.zero_()
    s_tmp = torch.zeros(1, device="cuda")
    ms_quant = _time_region(lambda: fq.quantize(x, fq.E4M3, layer.xq, s_tmp, layer.ws), it)
    del y_tmp

    flops_fwd = 2.0 * T * n * m
    # one plain device-to-device copy of known size: the reference that scales the FETCH_SIZE /
    # WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    calib = torch.empty_like(x)
    calib.copy_(x)
    torch.cuda.synchronize()
    del calib
    flops_dx = 2.0 * T * m * n
    flops_db = 2.0 * T * m * r
    tflops_fwd = flops_fwd / (ms_gemm_fwd * 1e-3) / 1e12
    tflops_dx = flops_dx / (ms_gemm_dx * 1e-3) / 1e12
    quant_bytes = 3.0 * T * n                      # read bf16 once (second read is cache-served), write FP8
    upd_bytes = 4.0 * m * r + 2.0 * k * n + r * n + 8.0 * k * r   # scores + selected rows in/out + adapter rows + buffer rows
    # The backbone product launched on its own.  Inside falqon_melded_fwd the same tile code runs in
    # gemm_fwd_pair_kernel, one launch that also carries the adapter's split-K tiles (see kernels).
    roofline = {"bound": "mfma", "kernel": "gemm_fp8_kernel<2,2,4,4,false,0> (forward, X~ . W~^T, 256 tiles of 256x256)",
                "achieved": tflops_fwd, "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tflops_fwd / FP8_PEAK_TFLOPS, "traffic": GEMM_FWD_TRAFFIC_BYTES,
                "flops_per_launch": flops_fwd, "avg_launch_ms": ms_gemm_fwd}
    if not args.no_context:
        roofline["same_launch_constant_operands"] = {
            "ms": ms_gemm_const, "TFLOP/s": flops_fwd / (ms_gemm_const * 1e-3) / 1e12,
            "frac": flops_fwd / (ms_gemm_const * 1e-3) / 1e12 / FP8_PEAK_TFLOPS,
            "note": "same kernel, grid and traffic with all codes = 1.0: the clock stays at its nominal value; the gap "
                    "to 'achieved' is the clock the chip grants for the workload's operand bits"}
        roofline["register_only_mfma_loop"] = {
            "TFLOP/s": tflops_probe, "ms": ms_probe, "frac_of_peak": tflops_probe / FP8_PEAK_TFLOPS,
            "achieved_over_loop": tflops_fwd / tflops_probe,
            "note": "same instruction count as the product, operands = this workload's FP8 codes held in registers, "
                    "no LDS/cache/HBM traffic: what the chip's power management lets the matrix cores sustain"}
    kernels = {
        "gemm_fwd": {"ms": ms_gemm_fwd, "TFLOP/s": tflops_fwd, "frac_fp8_peak": tflops_fwd / FP8_PEAK_TFLOPS},
        "gemm_dx": {"ms": ms_gemm_dx, "TFLOP/s": tflops_dx, "frac_fp8_peak": tflops_dx / FP8_PEAK_TFLOPS},
        "quantize_x": {"ms": ms_quant, "GB/s": quant_bytes / (ms_quant * 1e-3) / 1e9,
                       "frac_hbm_peak": quant_bytes / (ms_quant * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "proxy_update": {"ms": ms_upd, "GB/s": upd_bytes / (ms_upd * 1e-3) / 1e9,
                         "frac_hbm_peak": upd_bytes / (ms_upd * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "note": "three dependent launches over 1.6 MB: latency bound"},
        "adamw_buffer_step": {"grad_sqnorm_ms": ms_sqnorm, "adamw_delta_ms": ms_adamw,
                              "bytes": 28.0 * m * r, "GB/s": 28.0 * m * r / (ms_adamw * 1e-3) / 1e9,
                              "note": "optional replacement of the SGD buffer step inside melded_bwd; not in the timed step"},
        "db_bf16_variant": {"ms": ms_db_wide, "flops": flops_db,
                            "note": "dB = dy~^T O_A with O_A kept in bf16 (bf16 matrix cores), partial pass + ordered sum as "
                                    "two launches of their own; not in the timed step"},
        "fwd_after_quantize": {"ms_derived": ms_fwd - ms_quant, "flops": 2.0 * T * n * (m + r),
                               "TFLOP/s": 2.0 * T * n * (m + r) / ((ms_fwd - ms_quant) * 1e-3) / 1e12,
                               "note": "melded_fwd minus the quantizer: gemm_fwd_pair_kernel (backbone tiles + adapter "
                                       "split-K tiles in one launch) + the ordered sum of the adapter partials"},
        "bwd_after_quantize": {"ms_derived": ms_bwd - ms_quant, "flops": flops_dx + flops_db,
                               "TFLOP/s": (flops_dx + flops_db) / ((ms_bwd - ms_quant) * 1e-3) / 1e12,
                               "note": "melded_bwd minus the quantizer (E5M2 pass costs what the E4M3 pass does): "
                                       "gemm_dx_db_pair_kernel + the ordered sum of the dB partials with the buffer step"},
        "all_products": {"flops": 2.0 * T * n * (m + r) + flops_dx + flops_db,
                         "ms_derived": ms_fwd + ms_bwd - 2.0 * ms_quant,
                         "TFLOP/s": (2.0 * T * n * (m + r) + flops_dx + flops_db) / ((ms_fwd + ms_bwd - 2.0 * ms_quant) * 1e-3) / 1e12,
                         "frac_fp8_peak": (2.0 * T * n * (m + r) + flops_dx + flops_db) / ((ms_fwd + ms_bwd - 2.0 * ms_quant) * 1e-3) / 1e12 / FP8_PEAK_TFLOPS,
                         "note": "the three products of a step (forward with adapter columns, dX, dB) over everything "
                                 "in the two calls except the quantizer passes"},
        "calls": {"melded_fwd_ms": ms_fwd, "melded_bwd_ms": ms_bwd, "proxy_update_ms": ms_upd},
        "gemm_flops": {"fwd_backbone": flops_fwd, "fwd_adapter": 2.0 * T * n * r, "dx": flops_dx, "db": flops_db},
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
                               "fwd + bwd + proxy update per step"},
        "roofline": roofline, "kernels": kernels, "context": context,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, d, min(args.cpu_sample_tokens, T), args.cpu_reps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
