"""Swap the linear layers of an existing PyTorch model for melded layers, and step them together.

Python plumbing only: every computation is a C-ABI call made by `MeldedLoRALinear`.

    layers = meld_linears(model, rank=64, top_k=lambda m: m // 10)
    opt = MeldedOptimizer(layers, lr=2e-4)
    loss.backward(); opt.step()

`meld_linears` runs the initialization algorithm on each selected `nn.Linear` (quantize the weight,
rank-r factor of the quantization residual, adapter cast with the backbone's scale) and replaces the
module in place.  `MeldedOptimizer.step` is the loop body of the backward-and-update algorithm after
the gradients exist: global gradient norm over all layers, AdamW into every proxy buffer, then the
top-k fold of every layer.
"""
from typing import Callable, Iterable, List, Optional, Sequence, Union

import torch

from .nn import MeldedLoRALinear

LLAMA_PROJECTIONS = ("q_proj", "k_proj", "v_proj", "o_proj", "gate_proj", "up_proj", "down_proj")


class _WithBias(torch.nn.Module):
    """A melded layer followed by the original layer's (frozen) bias."""

    def __init__(self, layer: MeldedLoRALinear, bias: torch.Tensor):
        super().__init__()
        self.layer = layer
        self.register_buffer("bias", bias.detach().clone())

    def forward(self, x):
        y = self.layer(x)
        return y + self.bias.to(y.dtype)


def meld_linears(model: torch.nn.Module, rank: int = 64, top_k: Union[int, Callable[[int], int]] = 32,
                 names: Sequence[str] = LLAMA_PROJECTIONS, sgd_lr: Optional[float] = None, iters: int = 6,
                 seed: int = 0) -> List[MeldedLoRALinear]:
    """Replace every `nn.Linear` whose attribute name is in `names`; returns the new layers in module order.
    `top_k` is a row count or a function of the layer's output width.  Layers whose sizes the kernels do
    not take (widths not multiples of 16) raise."""
    made: List[MeldedLoRALinear] = []
    for parent in list(model.modules()):
        for child_name, child in list(parent.named_children()):
            if child_name not in names or not isinstance(child, torch.nn.Linear):
                continue
            m, n = child.out_features, child.in_features
            if m % 16 or n % 16:
                raise ValueError(f"{child_name}: {m}x{n} is not a multiple of 16 in both widths")
            k = top_k(m) if callable(top_k) else int(top_k)
            k = max(1, min(m, k))
            dev = child.weight.device
            if dev.type != "cuda":
                raise ValueError("move the model to the GPU before melding it")
            layer = MeldedLoRALinear(n, m, rank, k, sgd_lr=sgd_lr, device=dev)
            layer.init_from_weight(child.weight.detach(), iters=iters, seed=seed + len(made))
            made.append(layer)
            setattr(parent, child_name, layer if child.bias is None else _WithBias(layer, child.bias))
    return made


class MeldedOptimizer:
    """AdamW on the adapter gradients of a set of melded layers, written into their proxy buffers with one
    gradient-norm clip over all of them, followed by each layer's top-k fold every `fold_every` steps."""

    def __init__(self, layers: Iterable[MeldedLoRALinear], lr: float = 2e-4, betas=(0.9, 0.999), eps: float = 1e-8,
                 max_norm: float = 0.3, fold_every: int = 1):
        self.layers = list(layers)
        if not self.layers:
            raise ValueError("no melded layers")
        for l in self.layers:
            if l.sgd_lr is not None:
                raise ValueError("layers built with sgd_lr take their buffer step inside backward; use sgd_lr=None")
        self.lr, self.betas, self.eps, self.max_norm, self.fold_every = lr, betas, eps, max_norm, fold_every
        self.steps = 0
        self._sum_sq = torch.zeros(1, dtype=torch.float64, device=self.layers[0].wq.device)

    @torch.no_grad()
    def step(self) -> None:
        """Layers whose backward did not run since the last step have no gradient: like a parameter
        without `.grad` in a PyTorch optimizer they are left out of the norm and take no AdamW step
        (their moments do not decay either).  If no layer has one, that is an error: most likely the
        loss does not depend on the melded layers."""
        live = [l for l in self.layers if l.backward_calls > 0]
        if not live:
            raise RuntimeError("no melded layer received a gradient since the last step")
        self.steps += 1
        self._sum_sq.zero_()
        for l in live:
            l.grad_sqnorm(self._sum_sq)
        for l in live:
            l.adamw_step(self.steps, self._sum_sq, self.lr, self.betas[0], self.betas[1], self.eps, self.max_norm)
        if self.steps % self.fold_every == 0:
            for l in self.layers:
                l.proxy_update()
