"""The melded layer as a PyTorch module: autograd plumbing around the C-ABI calls.

Nothing of the method is computed here.  `MeldedLoRALinear.forward` calls `falqon_melded_fwd`, its
autograd backward calls `falqon_melded_bwd`, and `proxy_update()` / `adamw_step()` call the update
entry points.  The module owns the layer's persistent state (concatenated FP8 weight, its scale, the
proxy buffer) and a workspace; per-call outputs are fresh tensors, so a layer may be applied several
times before its backward passes run.

Where the adapter gradient goes: with an SGD rate (`sgd_lr`) every backward call takes the buffer
step itself, so calls add up in the proxy buffer.  Without one (`sgd_lr=None`, the optimizer path)
every backward call adds its gradient to `grad_acc` (the same call with the accumulator in the
buffer's place and a rate of -1: `acc += -(-1) * dB`), `d_b` holds the last call's gradient, and
`adamw_step()` consumes and clears the accumulator; `backward_calls` counts the calls since then.

The layer's only differentiable state is the proxy buffer, which autograd does not see.  So that the
backward pass runs even when the layer's input carries no gradient (the first projections behind a
frozen embedding), every layer owns a one-element parameter that is passed through the autograd
function as an anchor; it receives no gradient.  In that case the input-gradient product is skipped.
"""
from typing import Optional

import torch

from . import binding as _b


def _flat_bf16(t: torch.Tensor, width: int) -> torch.Tensor:
    t2 = t.reshape(-1, width)
    if t2.dtype != torch.bfloat16:
        t2 = t2.to(torch.bfloat16)
    return t2.contiguous()


def _layer_backward(layer: "MeldedLoRALinear", dy2: torch.Tensor, o_a, amax_oa, want_dx: bool):
    """One falqon_melded_bwd call; returns dx (None when the input needs no gradient)."""
    T, dev = dy2.shape[0], dy2.device
    dyq = torch.empty(T, layer.out_features, dtype=torch.uint8, device=dev)
    s_dy = torch.empty(1, dtype=torch.float32, device=dev)
    dx = torch.empty(T, layer.in_features, dtype=torch.bfloat16, device=dev) if want_dx else None
    if layer.sgd_lr is not None:
        buf, lr = layer.delta_buf, layer.sgd_lr            # the buffer step happens inside the call
    else:
        buf, lr = layer.grad_acc, -1.0                      # acc += dB, waiting for adamw_step()
    _b.melded_bwd(dy2, layer.wq, layer.s_w, o_a, amax_oa, layer.in_features, layer.rank, dyq, s_dy, dx,
                  layer.d_b, buf, lr, layer._workspace(T))
    layer.backward_calls += 1
    return dx


class _MeldedFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x: torch.Tensor, anchor: torch.Tensor, layer: "MeldedLoRALinear") -> torch.Tensor:
        lead = x.shape[:-1]
        x2 = _flat_bf16(x, layer.in_features)
        T = x2.shape[0]
        dev = x2.device
        ws = layer._workspace(T)
        xq = torch.empty(T, layer.in_features, dtype=torch.uint8, device=dev)
        s_x = torch.empty(1, dtype=torch.float32, device=dev)
        y = torch.empty(T, layer.out_features, dtype=torch.bfloat16, device=dev)
        o_a = torch.empty(T, layer.rank, dtype=torch.bfloat16, device=dev)
        amax_oa = torch.empty(1, dtype=torch.float32, device=dev)
        _b.melded_fwd(x2, layer.wq, layer.s_w, layer.out_features, layer.rank, xq, s_x, y, o_a, amax_oa, ws)
        ctx.layer, ctx.T, ctx.lead = layer, T, lead
        ctx.save_for_backward(o_a, amax_oa)
        return y.reshape(*lead, layer.out_features)

    @staticmethod
    def backward(ctx, dy: torch.Tensor):
        layer = ctx.layer
        o_a, amax_oa = ctx.saved_tensors
        dx = _layer_backward(layer, _flat_bf16(dy, layer.out_features), o_a, amax_oa, ctx.needs_input_grad[0])
        return (dx.reshape(*ctx.lead, layer.in_features) if dx is not None else None), None, None


class _MeldedGroupFn(torch.autograd.Function):
    """Several layers that read the same activation: the input is quantized once, every layer's
    product runs on those codes, and the input gradients are added."""

    @staticmethod
    def forward(ctx, x: torch.Tensor, anchor: torch.Tensor, group: "MeldedGroup"):
        layers = group.layers
        first = layers[0]
        lead = x.shape[:-1]
        x2 = _flat_bf16(x, first.in_features)
        T, dev = x2.shape[0], x2.device
        xq = torch.empty(T, first.in_features, dtype=torch.uint8, device=dev)
        s_x = torch.empty(1, dtype=torch.float32, device=dev)
        _b.quantize(x2, _b.E4M3, xq, s_x, first._workspace(T))
        outs, saved = [], []
        for layer in layers:
            y = torch.empty(T, layer.out_features, dtype=torch.bfloat16, device=dev)
            o_a = torch.empty(T, layer.rank, dtype=torch.bfloat16, device=dev)
            amax_oa = torch.empty(1, dtype=torch.float32, device=dev)
            _b.melded_fwd(None, layer.wq, layer.s_w, layer.out_features, layer.rank, xq, s_x, y, o_a, amax_oa,
                          layer._workspace(T))
            outs.append(y.reshape(*lead, layer.out_features))
            saved += [o_a, amax_oa]
        ctx.group, ctx.T, ctx.lead = group, T, lead
        ctx.save_for_backward(*saved)
        return tuple(outs)

    @staticmethod
    def backward(ctx, *dys):
        layers, T = ctx.group.layers, ctx.T
        saved = ctx.saved_tensors
        want_dx = ctx.needs_input_grad[0]
        total = None
        for i, (layer, dy) in enumerate(zip(layers, dys)):
            o_a, amax_oa = saved[2 * i], saved[2 * i + 1]
            if dy is None:
                dy2 = torch.zeros(T, layer.out_features, dtype=torch.bfloat16, device=o_a.device)
            else:
                dy2 = _flat_bf16(dy, layer.out_features)
            dx = _layer_backward(layer, dy2, o_a, amax_oa, want_dx)
            if want_dx:
                total = dx if total is None else total.add_(dx)
        return (total.reshape(*ctx.lead, layers[0].in_features) if want_dx else None), None, None


class MeldedGroup:
    """Melded layers with a common input (q/k/v, gate/up).  `group(x)` returns one output per layer."""

    def __init__(self, *layers: "MeldedLoRALinear"):
        if not layers or any(l.in_features != layers[0].in_features for l in layers):
            raise ValueError("a group needs layers of one input width")
        self.layers = list(layers)

    def __call__(self, x: torch.Tensor):
        return _MeldedGroupFn.apply(x, self.layers[0]._anchor, self)


class MeldedLoRALinear(torch.nn.Module):
    """y = x W'^T with W' the FP8 backbone that already contains the adapter; trainable only through
    the proxy buffer.  `sgd_lr` set: backward applies `DeltaBuffer += -lr dB` itself.  `sgd_lr=None`:
    backward adds dB to `grad_acc`; call `adamw_step()` (after `grad_sqnorm()` over all layers if the
    gradient norm is clipped), then `proxy_update()` at the chosen cadence."""

    def __init__(self, in_features: int, out_features: int, rank: int, top_k: int, sgd_lr: Optional[float] = 2e-4,
                 device="cuda"):
        super().__init__()
        self.in_features, self.out_features, self.rank, self.top_k = in_features, out_features, rank, top_k
        self.sgd_lr = sgd_lr
        dev = torch.device(device)
        self.register_buffer("wq", torch.zeros(out_features + rank, in_features, dtype=torch.uint8, device=dev))
        self.register_buffer("s_w", torch.ones(1, dtype=torch.float32, device=dev))
        self.register_buffer("delta_buf", torch.zeros(out_features, rank, dtype=torch.float32, device=dev))
        self.d_b = torch.zeros(out_features, rank, dtype=torch.float32, device=dev)       # the last backward call's dB
        self.grad_acc = (torch.zeros(out_features, rank, dtype=torch.float32, device=dev)
                         if sgd_lr is None else None)                                         # sum of dB since adamw_step()
        self.backward_calls = 0
        self.idx = torch.zeros(top_k, dtype=torch.int32, device=dev)
        self.exp_avg = None
        self.exp_avg_sq = None
        self.btq = None                 # B^T as E4M3 codes [r, m] and its scale: only for the A-update variant
        self.s_b = None
        self._ws = None
        # keeps autograd's backward running when the input carries no gradient; never receives one itself
        self._anchor = torch.nn.Parameter(torch.zeros(1, dtype=torch.float32, device=dev))

    def _workspace(self, T: int) -> torch.Tensor:
        """A workspace of at least the bytes this token count needs (the size is not monotonic in T,
        so it is asked for on every call and the buffer only ever grows)."""
        nbytes = _b.workspace_bytes(T, self.in_features, self.out_features, self.rank)
        if nbytes == 0:
            raise ValueError("invalid layer shape")
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device=self.wq.device)
        return self._ws

    @torch.no_grad()
    def load_weights(self, w: torch.Tensor, a: torch.Tensor) -> None:
        """W~, s_w <- Q(W); A~ <- cast(A * s_w); buffer <- 0 (the initialization steps after the SVD)."""
        ws = self._workspace(16)
        s_tmp = torch.zeros(1, dtype=torch.float32, device=self.wq.device)
        _b.quantize(w.float().contiguous(), _b.E4M3, self.wq[: self.out_features], self.s_w, ws)
        _b.quantize(a.float().contiguous(), _b.E4M3, self.wq[self.out_features:], s_tmp, ws, scale_in=self.s_w)
        self.delta_buf.zero_()

    @torch.no_grad()
    def init_from_weight(self, w: torch.Tensor, iters: int = 6, seed: int = 0, keep_left_factor: bool = False) -> torch.Tensor:
        """The whole initialization algorithm on the GPU: W~, s_w <- Q(W); E = DQ(W~) - W;
        A^ <- right factor of the rank-r SVD of E; A~ <- cast(A^ * s_w); buffer <- 0.
        Returns the Ritz values (approximate leading singular values of E).
        keep_left_factor: also keep B^ (transposed, cast to E4M3 with a scale of its own) in `btq`, `s_b`;
        only the variant that forms the gradient of A (binding.da) reads it."""
        dev = self.wq.device
        m, n, r = self.out_features, self.in_features, self.rank
        w32 = w.to(device=dev, dtype=torch.float32).contiguous()
        ws = self._workspace(16)
        _b.quantize(w32, _b.E4M3, self.wq[:m], self.s_w, ws)
        e = torch.empty(m, n, dtype=torch.float32, device=dev)
        _b.init_residual(w32, self.wq[:m], self.s_w, e)
        omega = torch.randn(r + 8, n, device=dev, generator=torch.Generator(device=dev).manual_seed(seed))
        a_hat = torch.empty(r, n, dtype=torch.float32, device=dev)
        sigma = torch.empty(r, dtype=torch.float32, device=dev)
        svd_ws = torch.empty(_b.svd_workspace_bytes(m, n, r), dtype=torch.uint8, device=dev)
        bt = torch.empty(r, m, dtype=torch.float32, device=dev) if keep_left_factor else None
        _b.svd_right_factor(e, r, omega, iters, a_hat, sigma, svd_ws, bt_out=bt)
        s_tmp = torch.zeros(1, dtype=torch.float32, device=dev)
        _b.quantize(a_hat, _b.E4M3, self.wq[m:], s_tmp, ws, scale_in=self.s_w)
        if keep_left_factor:
            self.btq = torch.empty(r, m, dtype=torch.uint8, device=dev)
            self.s_b = torch.zeros(1, dtype=torch.float32, device=dev)
            _b.quantize(bt, _b.E4M3, self.btq, self.s_b, ws)
        self.delta_buf.zero_()
        return sigma

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        return _MeldedFn.apply(x, self._anchor, self)

    def _accumulated(self) -> torch.Tensor:
        if self.grad_acc is None:
            raise RuntimeError("this layer takes its buffer step inside backward (sgd_lr is set); "
                               "build it with sgd_lr=None for the optimizer path")
        return self.grad_acc

    @torch.no_grad()
    def grad_sqnorm(self, sum_sq: torch.Tensor) -> None:
        """*sum_sq += squared norm of the gradient accumulated since the last adamw_step()."""
        _b.grad_sqnorm(self._accumulated(), sum_sq, self._workspace(16))

    @torch.no_grad()
    def adamw_step(self, step: int, sum_sq: Optional[torch.Tensor] = None, lr: float = 2e-4, beta1: float = 0.9,
                   beta2: float = 0.999, eps: float = 1e-8, max_norm: float = 0.3) -> None:
        """AdamW on the accumulated gradient into the proxy buffer; clears the accumulator."""
        g = self._accumulated()
        if self.exp_avg is None:
            self.exp_avg = torch.zeros_like(g)
            self.exp_avg_sq = torch.zeros_like(g)
        _b.adamw_delta(g, self.exp_avg, self.exp_avg_sq, self.delta_buf, step, lr, beta1, beta2, eps, sum_sq,
                       max_norm)
        g.zero_()
        self.backward_calls = 0

    @torch.no_grad()
    def proxy_update(self, clear_selected: bool = True) -> torch.Tensor:
        _b.proxy_update(self.delta_buf, self.wq, self.out_features, self.rank, self.top_k, self.idx,
                        self._workspace(16), clear_selected)
        return self.idx


class _RMSNorm(torch.nn.Module):
    def __init__(self, d: int, device="cuda"):
        super().__init__()
        self.weight = torch.nn.Parameter(torch.ones(d, dtype=torch.bfloat16, device=device), requires_grad=False)

    def forward(self, x):
        v = x.float()
        return (v * torch.rsqrt(v.pow(2).mean(-1, keepdim=True) + 1e-5)).to(x.dtype) * self.weight


class LlamaBlock(torch.nn.Module):
    """One LLaMA decoder block whose seven projections are melded layers (q, k, v, o, gate, up,
    down); normalisation, attention and the SwiGLU product are plain PyTorch operations, there only
    to put real data dependence between the projections.  `linear(in, out)` builds a projection, so
    the same block can be instantiated with another linear layer for comparison."""

    def __init__(self, d_model: int, n_heads: int, d_mlp: int, linear, device="cuda", share_quantized_inputs: bool = True):
        super().__init__()
        self.n_heads = n_heads
        self.norm1, self.norm2 = _RMSNorm(d_model, device), _RMSNorm(d_model, device)
        self.q, self.k, self.v, self.o = (linear(d_model, d_model) for _ in range(4))
        self.gate, self.up = linear(d_model, d_mlp), linear(d_model, d_mlp)
        self.down = linear(d_mlp, d_model)
        # melded projections that share an input quantize it once
        melded = all(isinstance(p, MeldedLoRALinear) for p in self.projections())
        self._qkv = MeldedGroup(self.q, self.k, self.v) if melded and share_quantized_inputs else None
        self._gate_up = MeldedGroup(self.gate, self.up) if melded and share_quantized_inputs else None

    def forward(self, x):                                              # x: [batch, seq, d_model] bf16
        B, S, D = x.shape
        h = self.norm1(x)
        qkv = self._qkv(h) if self._qkv is not None else (self.q(h), self.k(h), self.v(h))
        q, k, v = (t.reshape(B, S, self.n_heads, D // self.n_heads).transpose(1, 2) for t in qkv)
        a = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
        x = x + self.o(a.transpose(1, 2).reshape(B, S, D))
        h = self.norm2(x)
        gate, up = self._gate_up(h) if self._gate_up is not None else (self.gate(h), self.up(h))
        return x + self.down(torch.nn.functional.silu(gate) * up)

    def projections(self):
        return [self.q, self.k, self.v, self.o, self.gate, self.up, self.down]
