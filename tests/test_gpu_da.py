"""The A-update variant on the GPU: gradient of the adapter factor A against the oracle, and the left
factor of the initialization against the oracle's exact SVD."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
import workloads
from gpu_common import layer_on_gpu, np_of, oracle_weights, relf

pytestmark = pytest.mark.gpu


def _run_da(dyq, s_dy, btq, s_b, xq, s_x):
    T, m = dyq.shape
    n, r = xq.shape[1], btq.shape[0]
    dev = "cuda"
    g = torch.full((T, r), float("nan"), dtype=torch.bfloat16, device=dev)
    amax = torch.zeros(1, device=dev)
    d_at = torch.full((n, r), float("nan"), device=dev)
    ws = torch.empty(fq.workspace_bytes(T, m, n, r), dtype=torch.uint8, device=dev)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    sc = lambda v: torch.tensor([v], dtype=torch.float32, device=dev)
    fq.da(t(dyq), sc(s_dy), t(btq), sc(s_b), t(xq), sc(s_x), g, amax, d_at, ws)
    torch.cuda.synchronize()
    return np_of(g), np.float32(amax.item()), np_of(d_at)


@pytest.mark.parametrize("T,n,m,r", [(256, 512, 512, 16), (200, 384, 208, 48), (1, 128, 16, 16), (2100, 1040, 4112, 64),
                                     (700, 272, 528, 128)])
def test_gradient_of_a_matches_the_oracle(T, n, m, r):
    d = workloads.make_inputs(T, n, m, r, seed=9100 + T, outliers=True)
    xq, s_x, _ = oracle.quantize(d["x"].float().numpy(), oracle.E4M3)
    dyq, s_dy, _ = oracle.quantize(d["dy"].float().numpy(), oracle.E5M2)
    bt = (np.random.default_rng(T).normal(size=(r, m)) * 0.05).astype(np.float32)
    btq, s_b, _ = oracle.quantize(bt, oracle.E4M3)
    print(f"dA T={T} n={n} m={m} r={r}", flush=True)
    g, amax, d_at = _run_da(dyq, s_dy, btq, s_b, xq, s_x)
    g_ref = oracle.adapter_inner_grad(dyq, s_dy, btq, s_b)
    assert relf(g, g_ref) < 1e-3                                     # fp32 accumulation against fp64, both rounded to bf16
    assert np.max(np.abs(g - g_ref)) <= 2.0 ** -7 * np.max(np.abs(g_ref))
    assert amax == np.max(np.abs(g))
    # the second product on the GPU's own g: nothing is rounded before the fp32 accumulation
    ref = oracle.da(xq, s_x, g)
    assert relf(d_at, ref) < 1e-5
    assert relf(d_at, oracle.da(xq, s_x, g_ref)) < 2e-3              # and the whole call against the whole oracle


def test_gradient_of_a_exact_integer_case_is_bit_exact():
    g = np.random.default_rng(11)
    T, n, m, r = 300, 272, 400, 32
    X = g.integers(-3, 4, size=(T, n)).astype(np.float32)
    dY = g.integers(-2, 3, size=(T, m)).astype(np.float32)
    Bt = g.integers(-2, 3, size=(r, m)).astype(np.float32)
    xq = oracle.fp8_encode(X * 4, oracle.E4M3)
    dyq = oracle.fp8_encode(dY * 8, oracle.E5M2)
    btq = oracle.fp8_encode(Bt * 2, oracle.E4M3)
    gg, amax, d_at = _run_da(dyq, np.float32(8.0), btq, np.float32(2.0), xq, np.float32(4.0))
    G = dY.astype(np.float64) @ Bt.T.astype(np.float64)
    assert np.max(np.abs(G)) < 256                                    # exact in bf16
    assert np.array_equal(gg.astype(np.float64), G)
    assert np.array_equal(d_at.astype(np.float64), X.T.astype(np.float64) @ G)
    assert amax == np.max(np.abs(G))


def test_left_factor_of_the_initialization():
    """bt_out^T a_out is the rank-r part of E; rows of bt_out are orthogonal with squared norms sigma."""
    g = np.random.default_rng(12)
    m, n, r = 384, 512, 16
    U, _ = np.linalg.qr(g.normal(size=(m, m)))
    V, _ = np.linalg.qr(g.normal(size=(n, n)))
    sv = np.concatenate([np.linspace(8, 2, r), np.full(m - r, 1e-3)])
    E = ((U * sv[None, :]) @ V[:m]).astype(np.float32)
    e = torch.from_numpy(E).cuda()
    omega = torch.randn(r + 8, n, device="cuda", generator=torch.Generator(device="cuda").manual_seed(1))
    a = torch.empty(r, n, device="cuda")
    sg = torch.empty(r, device="cuda")
    bt = torch.empty(r, m, device="cuda")
    ws = torch.empty(fq.svd_workspace_bytes(m, n, r), dtype=torch.uint8, device="cuda")
    fq.svd_right_factor(e, r, omega, 6, a, sg, ws, bt_out=bt)
    torch.cuda.synchronize()
    B, A, s = oracle.svd_factors(E, r)
    assert np.allclose(np_of(sg), s[:r], rtol=1e-4)
    assert relf(np_of(bt).T.astype(np.float64) @ np_of(a).astype(np.float64), B @ A) < 1e-3
    gram = np_of(bt).astype(np.float64) @ np_of(bt).astype(np.float64).T
    assert np.allclose(np.diag(gram), s[:r], rtol=1e-3)
    assert np.max(np.abs(gram - np.diag(np.diag(gram)))) < 1e-3 * s[0]


def test_variant_end_to_end_from_a_layer():
    """From the initialization to the gradient: B^ from the factorization, the layer's own x~ and dy~."""
    T, n, m, r = 320, 512, 640, 32
    w = (np.random.default_rng(13).normal(size=(m, n)) * 0.02).astype(np.float32)
    d = workloads.make_inputs(T, n, m, r, seed=9200)
    from paper_2510_24061_amd.nn import MeldedLoRALinear
    lin = MeldedLoRALinear(n, m, r, 8, sgd_lr=None)
    lin.init_from_weight(torch.from_numpy(w), iters=8, keep_left_factor=True)
    assert lin.btq is not None and lin.btq.shape == (r, m)
    layer = fq.MeldedLinear(T, n, m, r, 8)
    layer.wq.copy_(lin.wq); layer.s_w.copy_(lin.s_w)
    layer.forward(d["x"].cuda()); layer.backward(d["dy"].cuda(), accumulate=False)
    g = torch.empty(T, r, dtype=torch.bfloat16, device="cuda")
    amax = torch.zeros(1, device="cuda")
    d_at = torch.empty(n, r, device="cuda")
    ws = torch.empty(fq.workspace_bytes(T, m, n, r), dtype=torch.uint8, device="cuda")
    fq.da(layer.dyq, layer.s_dy, lin.btq, lin.s_b, layer.xq, layer.s_x, g, amax, d_at, ws)
    torch.cuda.synchronize()
    g_ref = oracle.adapter_inner_grad(np_of(layer.dyq), np.float32(layer.s_dy.item()), np_of(lin.btq), np.float32(lin.s_b.item()))
    assert relf(np_of(g), g_ref) < 1e-3
    assert relf(np_of(d_at), oracle.da(np_of(layer.xq), np.float32(layer.s_x.item()), np_of(g))) < 1e-5
    assert np.isfinite(np_of(d_at)).all() and np.abs(np_of(d_at)).sum() > 0
