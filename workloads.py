"""Seeded synthetic inputs for the melded FP8-LoRA layer.

Shared by the CPU oracle's tests and the GPU path's tests and benchmark.  It
holds no arithmetic of the method: it only draws random tensors with the
shapes and value structure of the paper's workloads (LLaMA-7B / 13B linear
projections under LoRA fine-tuning, rank 64; "Experimental settings").
Those weights and datasets are not available, so every tensor is synthetic:

  X   bf16 [T, n]   ~ N(0, 1); for the LLaMA-shaped configs round(0.01 n)
                    channels (a seeded choice) are multiplied by 20, standing
                    in for the outlier channels of LLM activations
  W   fp32 [m, n]   ~ N(0, std 0.02)
  A   fp32 [r, n]   ~ N(0, std 1/r)
  dY  bf16 [T, m]   ~ N(0, 1)
  B = 0 is implicit (the proxy buffer starts at zero).

All draws are fp32 from a torch.Generator and are cast once.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import torch

BASE_SEED = 20251024


@dataclass(frozen=True)
class LayerShape:
    name: str
    m: int          # out features
    n: int          # in features
    count: int = 1  # how many such projections the config holds


@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    T: int
    r: int
    k: int
    outliers: bool
    layers: Tuple[LayerShape, ...]
    lr: float = 2e-4
    accumulate_steps: int = 1


CONFIGS = {
    1: Config(1, "single-512", 256, 16, 8, False, (LayerShape("lin", 512, 512),)),
    2: Config(2, "llama7b-attn", 4096, 64, 32, True, (LayerShape("attn", 4096, 4096),)),
    3: Config(3, "llama7b-mlp", 4096, 64, 32, True,
              (LayerShape("up", 11008, 4096), LayerShape("down", 4096, 11008))),
    4: Config(4, "llama13b-block", 8192, 64, 64, True,
              (LayerShape("attn", 5120, 5120, 4), LayerShape("up", 13824, 5120, 2),
               LayerShape("down", 5120, 13824, 1))),
    5: Config(5, "llama7b-stack", 4096, 64, 32, True,
              (LayerShape("attn", 4096, 4096, 128), LayerShape("up", 11008, 4096, 64),
               LayerShape("down", 4096, 11008, 32)), accumulate_steps=4),
}


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def make_inputs(T: int, n: int, m: int, r: int, seed: int, outliers: bool = False,
                x_std: float = 1.0, w_std: float = 0.02, dy_std: float = 1.0):
    """CPU tensors x (bf16), w (fp32), a (fp32), dy (bf16) for one layer."""
    g = _gen(seed)
    x = torch.randn(T, n, generator=g, dtype=torch.float32) * x_std
    if outliers and n > 0:
        n_out = max(1, round(0.01 * n))
        cols = torch.randperm(n, generator=g)[:n_out]
        x[:, cols] *= 20.0
    w = torch.randn(m, n, generator=g, dtype=torch.float32) * w_std
    a = torch.randn(r, n, generator=g, dtype=torch.float32) * (1.0 / max(r, 1))
    dy = torch.randn(T, m, generator=g, dtype=torch.float32) * dy_std
    return dict(x=x.to(torch.bfloat16), w=w, a=a, dy=dy.to(torch.bfloat16))


def config_layer_inputs(cfg: int, layer_index: int = 0):
    c = CONFIGS[cfg]
    shape = c.layers[layer_index]
    seed = BASE_SEED + 1000 * cfg + layer_index
    d = make_inputs(c.T, shape.n, shape.m, c.r, seed, c.outliers)
    d["shape"] = shape
    d["config"] = c
    return d


def make_delta_buffer(m: int, r: int, seed: int, scale: float = 2e-4, ties: bool = False):
    """A proxy buffer as some steps of accumulation would leave it: fp32 [m, r],
    entries ~ N(0, scale) with a per-row log-normal spread so that row scores differ
    by orders of magnitude.  With ties=True groups of rows are exact copies or sign
    flips of one another, which makes their scores equal."""
    g = _gen(seed)
    buf = torch.randn(m, r, generator=g, dtype=torch.float32) * scale
    row_scale = torch.exp(torch.randn(m, 1, generator=g, dtype=torch.float32))
    buf = buf * row_scale
    if ties and m >= 8:
        src = torch.randperm(m, generator=g)[: max(1, m // 8)]
        for s in src.tolist():
            for d in ((s * 7 + 3) % m, (s * 13 + 5) % m):
                buf[d] = -buf[s]
    return buf.contiguous()
