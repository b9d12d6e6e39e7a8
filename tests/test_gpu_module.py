"""The autograd wrapper: same bytes as the direct calls, gradients flow through a decoder block."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
import workloads
from paper_2510_24061_amd.nn import LlamaBlock, MeldedLoRALinear
from gpu_common import np_of, oracle_weights, relf

pytestmark = pytest.mark.gpu


def test_module_matches_direct_calls_and_oracle():
    T, n, m, r, k = 192, 256, 384, 32, 6
    d = workloads.make_inputs(T, n, m, r, seed=5150)
    wcat, s_w = oracle_weights(d["w"], d["a"])
    lin = MeldedLoRALinear(n, m, r, k, sgd_lr=2e-4)
    lin.load_weights(d["w"].cuda(), d["a"].cuda())
    torch.cuda.synchronize()
    assert np.array_equal(np_of(lin.wq), wcat) and np.float32(lin.s_w.item()).tobytes() == s_w.tobytes()

    x = d["x"].cuda().reshape(2, T // 2, n).requires_grad_(True)     # leading dimensions are flattened
    y = lin(x)
    y.backward(d["dy"].cuda().reshape(2, T // 2, m))
    lin.proxy_update()
    torch.cuda.synchronize()

    ref = fq.MeldedLinear(T, n, m, r, k)
    ref.wq.copy_(torch.from_numpy(wcat)); ref.s_w.fill_(float(s_w))
    ref.forward(d["x"].cuda()); ref.backward(d["dy"].cuda(), lr=2e-4); ref.update()
    torch.cuda.synchronize()
    assert np_of(y).reshape(T, m).tobytes() == np_of(ref.y).tobytes()
    assert np_of(x.grad).reshape(T, n).tobytes() == np_of(ref.dx).tobytes()
    assert np_of(lin.d_b).tobytes() == np_of(ref.d_b).tobytes()
    assert np_of(lin.wq).tobytes() == np_of(ref.wq).tobytes()
    assert np_of(lin.delta_buf).tobytes() == np_of(ref.delta_buf).tobytes()
    f = oracle.layer_fwd(d["x"].float().numpy(), wcat, s_w, m, r)
    assert relf(np_of(y).reshape(T, m), oracle.round_bf16(f["y"])) < 1e-3


def test_decoder_block_trains_through_the_buffers():
    """Forward and backward through a small block: every projection receives a gradient, fills its
    buffer, and the proxy update moves rows of every weight."""
    torch.manual_seed(0)
    d_model, heads, d_mlp, r, k = 256, 4, 688 // 16 * 16, 16, 8
    g = torch.Generator().manual_seed(3)

    def linear(i, o):
        lin = MeldedLoRALinear(i, o, r, k, sgd_lr=0.05)
        lin.load_weights((torch.randn(o, i, generator=g) * 0.05).cuda(), (torch.randn(r, i, generator=g) / r).cuda())
        return lin

    block = LlamaBlock(d_model, heads, d_mlp, linear)
    before = [p.wq.clone() for p in block.projections()]
    x = torch.randn(2, 64, d_model, generator=g).to(torch.bfloat16).cuda().requires_grad_(True)
    out = block(x)
    assert out.shape == x.shape and torch.isfinite(out.float()).all()
    out.float().pow(2).mean().backward()
    assert torch.isfinite(x.grad.float()).all() and x.grad.float().abs().sum() > 0
    for p, w0 in zip(block.projections(), before):
        assert p.delta_buf.abs().sum() > 0
        idx = p.proxy_update().clone()
        torch.cuda.synchronize()
        assert len(set(idx.tolist())) == k
        assert (p.wq[: p.out_features] != w0[: p.out_features]).any()
        assert (p.wq[p.out_features:] == w0[p.out_features:]).all()        # adapter rows are never written


def test_module_initializes_itself_from_a_weight():
    n, m, r, k = 512, 640, 32, 8
    w = (np.random.default_rng(8).normal(size=(m, n)) * 0.02).astype(np.float32)
    lin = MeldedLoRALinear(n, m, r, k)
    sigma = lin.init_from_weight(torch.from_numpy(w), iters=8)
    torch.cuda.synchronize()
    ref = oracle.init_adapter(w, r)
    assert np.array_equal(np_of(lin.wq[:m]), ref["wq"]) and np.float32(lin.s_w.item()).tobytes() == ref["s_w"].tobytes()
    sg = np_of(sigma).astype(np.float64)
    assert np.all(np.diff(sg) <= 0) and np.all(sg <= ref["sv"][:r] * (1 + 1e-4))
    assert np.sum(sg ** 2) >= 0.9 * np.sum(ref["sv"][:r] ** 2)
    # adapter rows: codes of a matrix with orthogonal rows of squared norm sigma_i, at the backbone's scale
    a = oracle.fp8_decode(np_of(lin.wq[m:]), oracle.E4M3) / np.float64(ref["s_w"])
    gram = a @ a.T
    assert np.max(np.abs(np.diag(gram) - sg)) <= 0.02 * sg[0]         # FP8 rounding of the entries
    off = gram - np.diag(np.diag(gram))
    assert np.max(np.abs(off)) <= 0.05 * sg[0]
    assert not lin.delta_buf.any()


def test_group_with_one_quantized_input_equals_the_separate_layers():
    from paper_2510_24061_amd.nn import MeldedGroup
    T, n, r = 320, 256, 16
    widths = (256, 128, 384)
    g = torch.Generator().manual_seed(77)
    x0 = torch.randn(T, n, generator=g).to(torch.bfloat16).cuda()
    dys = [torch.randn(T, m, generator=g).to(torch.bfloat16).cuda() for m in widths]

    def build():
        layers = []
        gg = torch.Generator().manual_seed(78)
        for m in widths:
            lin = MeldedLoRALinear(n, m, r, 8, sgd_lr=1e-3)
            lin.load_weights((torch.randn(m, n, generator=gg) * 0.02).cuda(), (torch.randn(r, n, generator=gg) / r).cuda())
            layers.append(lin)
        return layers

    sep, grp = build(), build()
    xs = x0.clone().requires_grad_(True)
    ys = [l(xs) for l in sep]
    torch.autograd.backward(ys, dys)
    xg = x0.clone().requires_grad_(True)
    yg = MeldedGroup(*grp)(xg)
    torch.autograd.backward(list(yg), dys)
    torch.cuda.synchronize()
    for a, b, ls, lg in zip(ys, yg, sep, grp):
        assert torch.equal(a, b)                                        # same codes, same product
        assert torch.equal(ls.d_b, lg.d_b) and torch.equal(ls.delta_buf, lg.delta_buf)
    # input gradient: the same three bf16 terms, possibly added in another order
    assert relf(np_of(xg.grad), np_of(xs.grad)) < 1e-2
    # a layer whose output is not used gets a zero gradient and still takes part
    xg2 = x0.clone().requires_grad_(True)
    y0, _, _ = MeldedGroup(*grp)(xg2)
    y0.backward(dys[0])
    xs2 = x0.clone().requires_grad_(True)
    sep[0](xs2).backward(dys[0])
    assert torch.equal(xg2.grad, xs2.grad)
    with pytest.raises(ValueError):
        MeldedGroup(grp[0], MeldedLoRALinear(128, 64, 16, 4))


def test_forward_call_accepts_an_already_quantized_input():
    T, n, m, r, k = 200, 128, 192, 16, 4
    d = workloads.make_inputs(T, n, m, r, seed=31)
    wcat, s_w = oracle_weights(d["w"], d["a"])
    a = fq.MeldedLinear(T, n, m, r, k)
    a.wq.copy_(torch.from_numpy(wcat)); a.s_w.fill_(float(s_w))
    a.forward(d["x"].cuda())
    b = fq.MeldedLinear(T, n, m, r, k)
    b.wq.copy_(a.wq); b.s_w.copy_(a.s_w)
    b.xq.copy_(a.xq); b.s_x.copy_(a.s_x)
    b.amax_oa.fill_(123.0)                                              # must be reset by the call
    fq.melded_fwd(None, b.wq, b.s_w, m, r, b.xq, b.s_x, b.y, b.o_a, b.amax_oa, b.ws)
    torch.cuda.synchronize()
    assert torch.equal(a.y, b.y) and torch.equal(a.o_a, b.o_a) and torch.equal(a.amax_oa, b.amax_oa)


def test_workspace_follows_the_bytes_needed_not_the_token_count():
    """The workspace size need not be monotonic in T (split counts change at tile boundaries): the
    module asks for the size on every call, so a layer that has seen one token count serves any other."""
    n = m = 4096
    r = 64
    g = torch.Generator().manual_seed(12)
    lin = MeldedLoRALinear(n, m, r, 8, sgd_lr=1e-3)
    lin.load_weights((torch.randn(m, n, generator=g) * 0.02).cuda(), (torch.randn(r, n, generator=g) / r).cuda())
    for T in (4200, 4096, 16, 4200):
        x = torch.randn(T, n, generator=g).to(torch.bfloat16).cuda().requires_grad_(True)
        y = lin(x)
        y.backward(torch.ones_like(y))
        torch.cuda.synchronize()
        assert torch.isfinite(x.grad.float()).all()
    lin.proxy_update()
    torch.cuda.synchronize()


def test_backward_runs_when_the_input_carries_no_gradient():
    """A layer behind frozen modules: its input does not require a gradient, its adapter gradient must
    still be formed (and be the one a call with an input gradient forms)."""
    T, n, m, r, k = 192, 256, 384, 32, 6
    d = workloads.make_inputs(T, n, m, r, seed=616)
    dy = d["dy"].cuda()
    a = MeldedLoRALinear(n, m, r, k, sgd_lr=None)
    a.load_weights(d["w"].cuda(), d["a"].cuda())
    b = MeldedLoRALinear(n, m, r, k, sgd_lr=None)
    b.load_weights(d["w"].cuda(), d["a"].cuda())
    x_frozen = d["x"].cuda()
    assert not x_frozen.requires_grad
    ya = a(x_frozen)
    assert ya.requires_grad
    ya.backward(dy)
    xb = d["x"].cuda().requires_grad_(True)
    b(xb).backward(dy)
    torch.cuda.synchronize()
    assert a.backward_calls == 1 and a._anchor.grad is None
    assert a.d_b.abs().sum() > 0
    assert torch.equal(a.d_b, b.d_b) and torch.equal(a.grad_acc, b.grad_acc)
    assert xb.grad is not None


def test_gradients_of_several_backward_calls_add_up():
    """Optimizer path: a layer applied twice in one graph, then a second micro-batch, before one
    optimizer step.  The accumulator holds the sum of the three gradients; the step clears it."""
    T, n, m, r, k = 128, 256, 272, 16, 6
    d = workloads.make_inputs(T, n, m, r, seed=617)
    lin = MeldedLoRALinear(n, m, r, k, sgd_lr=None)
    lin.load_weights(d["w"].cuda(), d["a"].cuda())
    x1 = d["x"].cuda().requires_grad_(True)
    x2 = (d["x"].cuda().float() * 0.5).to(torch.bfloat16).requires_grad_(True)
    dy = d["dy"].cuda()
    singles = []
    for x, g in ((x2, dy * 2), (x1, dy), (x1, dy * 3)):              # autograd runs the later use first
        ref = MeldedLoRALinear(n, m, r, k, sgd_lr=None)
        ref.wq.copy_(lin.wq); ref.s_w.copy_(lin.s_w)
        ref(x.detach()).backward(g)
        singles.append(ref.d_b.clone())
    y = lin(x1) + 2.0 * lin(x2)                                        # one graph, two uses
    y.backward(dy)
    lin(x1).backward(dy * 3)                                           # a second micro-batch
    torch.cuda.synchronize()
    assert lin.backward_calls == 3
    want = (singles[0] + singles[1]) + singles[2]
    alt = (singles[1] + singles[0]) + singles[2]
    assert torch.equal(lin.grad_acc, want) or torch.equal(lin.grad_acc, alt)
    ss = torch.zeros(1, dtype=torch.float64, device="cuda")
    lin.grad_sqnorm(ss)
    lin.adamw_step(1, ss)
    torch.cuda.synchronize()
    assert lin.backward_calls == 0 and not lin.grad_acc.any()
    assert lin.delta_buf.abs().sum() > 0
    ref_buf = oracle.adamw_delta(np_of(want), np.zeros((m, r), np.float32), np.zeros((m, r), np.float32),
                                 np.zeros((m, r), np.float32), 1,
                                 clip_coef=oracle.clip_coef(oracle.sum_squares(np_of(want)), 0.3))[2]
    assert relf(np_of(lin.delta_buf), ref_buf) < 1e-5
