"""GPU parity of the optimizer step into the proxy buffer (AdamW under gradient-norm clipping)
against the CPU oracle.

Bars.  The sum of squares is an fp64 sum in another order than the oracle's: relative 1e-12.
The step is computed in fp32 on the GPU and in fp64 (from the same fp32 state) by the oracle, so
each stored value may differ by the roundings of the fp32 operations that form it (unit
roundoff 6e-8 each).  A moment is a sum of two terms that may cancel: the first must agree to
4e-7 of its larger term, the second to 6e-7 (the clipped gradient carries two roundings and is
squared, which doubles them; three more operations follow: about seven roundings).  The change of the buffer, -(lr/bias1) * m / denom, inherits that absolute error
of m scaled by (lr/bias1)/denom, plus a few roundings of its own: 1e-6 of (lr/bias1) * term/denom
plus 1e-6 of the change.  The buffer itself adds one rounding (an ulp of its value).  Over the
whole tensor the change must agree to 2e-6 in relative Frobenius norm.
Every step is fed from the oracle's state, never from the previous GPU step."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
from gpu_common import np_of, relf

pytestmark = pytest.mark.gpu


def _gpu(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()


@pytest.mark.parametrize("count", [4, 256, 1000, 4096 * 64, 11008 * 64 + 4])
def test_grad_sqnorm(count):
    g = (np.random.default_rng(count).normal(size=count) * 3).astype(np.float32)
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    acc = torch.tensor([1.5], dtype=torch.float64, device="cuda")          # accumulates on top of what is there
    fq.grad_sqnorm(_gpu(g), acc, ws)
    fq.grad_sqnorm(_gpu(g), acc, ws)
    torch.cuda.synchronize()
    want = 1.5 + 2.0 * oracle.sum_squares(g)
    assert abs(acc.item() - want) <= 1e-12 * want
    acc2 = torch.tensor([1.5], dtype=torch.float64, device="cuda")
    fq.grad_sqnorm(_gpu(g), acc2, ws)
    fq.grad_sqnorm(_gpu(g), acc2, ws)
    torch.cuda.synchronize()
    assert acc2.item() == acc.item()                                        # reproducible


def _check_step(gr, m0, v0, b0, step, coef_ss, **hyper):
    """coef_ss: None (no clipping) or the squared global norm."""
    d_b, ea, es, buf = _gpu(gr), _gpu(m0), _gpu(v0), _gpu(b0)
    ss = None if coef_ss is None else torch.tensor([coef_ss], dtype=torch.float64, device="cuda")
    fq.adamw_delta(d_b, ea, es, buf, step, sum_sq=ss, **hyper)
    torch.cuda.synchronize()
    okw = {k: v for k, v in hyper.items() if k != "max_norm"}
    coef = 1.0 if coef_ss is None else oracle.clip_coef(coef_ss, hyper.get("max_norm", 0.3))
    m1, v1, b1 = oracle.adamw_delta(gr, m0, v0, b0, step, clip_coef=coef, **okw)
    gm, gv, gb = np_of(ea), np_of(es), np_of(buf)
    b1d, b2d = okw.get("beta1", 0.9), okw.get("beta2", 0.999)
    g64 = coef * gr.astype(np.float64)
    term_m = np.maximum(np.abs(b1d * m0.astype(np.float64)), np.abs((1 - b1d) * g64))
    term_v = np.maximum(b2d * v0.astype(np.float64), (1 - b2d) * g64 * g64)
    assert np.all(np.abs(gm - m1) <= 4e-7 * term_m + 1e-45)
    assert np.all(np.abs(gv - v1) <= 6e-7 * term_v + 1e-45)
    dg, do = gb.astype(np.float64) - b0, b1.astype(np.float64) - b0
    lr = okw.get("lr", 2e-4)
    denom = np.sqrt(v1.astype(np.float64)) / np.sqrt(1 - b2d ** step) + okw.get("eps", 1e-8)
    term_change = (lr / (1 - b1d ** step)) * term_m / denom
    ulp = np.spacing(np.maximum(np.abs(b1), np.abs(gb)).astype(np.float32)).astype(np.float64)   # binade edges
    assert np.all(np.abs(gb.astype(np.float64) - b1) <= 1e-6 * term_change + 1e-6 * np.abs(do) + ulp + 1e-45)
    small_buf = np.abs(b0) <= 4 * np.abs(do)         # elsewhere the change is only known to an ulp of the buffer
    if np.any(small_buf) and np.max(np.abs(do)) > 0:
        assert relf(dg[small_buf], do[small_buf]) < 2e-6
    return m1, v1, b1


@pytest.mark.parametrize("m,r", [(16, 16), (528, 48), (4096, 64), (13824, 64), (256, 256)])
def test_adamw_first_step_and_chain(m, r):
    g = np.random.default_rng(m + r)
    z = np.zeros((m, r), np.float32)
    state = (z, z, (g.normal(size=(m, r)) * 1e-4).astype(np.float32))
    for step in range(1, 5):
        gr = (g.normal(size=(m, r)) * [1e-3, 1.0, 1e-6, 50.0][step - 1]).astype(np.float32)
        ss = oracle.sum_squares(gr) * 3.0                                    # as if two more layers shared the norm
        print(f"adamw m={m} r={r} step={step}", flush=True)
        state = _check_step(gr, *state, step, ss if step % 2 == 0 else None)


def test_adamw_special_values_and_hyperparameters():
    m, r = 32, 16
    g = np.random.default_rng(1)
    gr = (g.normal(size=(m, r))).astype(np.float32)
    gr[0, :4] = [0.0, -0.0, 1e-30, -3e4]
    m0 = (g.normal(size=(m, r)) * 0.1).astype(np.float32)
    v0 = (g.normal(size=(m, r)) ** 2 * 0.01).astype(np.float32)
    m0[1, :2] = 0.0
    v0[1, :2] = 0.0
    b0 = (g.normal(size=(m, r))).astype(np.float32)
    _check_step(gr, m0, v0, b0, 7, None, lr=1e-2, beta1=0.8, beta2=0.95, eps=1e-6)
    _check_step(gr, m0, v0, b0, 1000, 1e-8, max_norm=0.3)                  # tiny norm: coefficient exactly 1
    _check_step(gr, m0, v0, b0, 3, 1e6, max_norm=1.0, lr=5e-3)             # heavy clipping
    # zero gradient, zero moments: nothing moves
    z = np.zeros((m, r), np.float32)
    d_b, ea, es, buf = _gpu(z), _gpu(z), _gpu(z), _gpu(b0)
    fq.adamw_delta(d_b, ea, es, buf, 1)
    torch.cuda.synchronize()
    assert np.array_equal(np_of(buf), b0) and not np_of(ea).any() and not np_of(es).any()


def test_training_loop_with_adamw_feeds_the_proxy_update():
    """bwd (no SGD step) -> global norm over two layers -> AdamW into the buffers -> proxy update,
    all on the GPU; the update applied to the GPU's own buffer must equal the oracle's applied to
    those bytes, and the buffers must match the oracle chain within the step's tolerance."""
    import workloads
    from gpu_common import layer_on_gpu, oracle_weights
    layers, refs = [], []
    ss = torch.zeros(1, dtype=torch.float64, device="cuda")
    for li, (T, n, m, r, k) in enumerate([(256, 512, 512, 16, 8), (192, 256, 384, 32, 6)]):
        d = workloads.make_inputs(T, n, m, r, seed=900 + li)
        wcat, s_w = oracle_weights(d["w"], d["a"])
        layer = layer_on_gpu(T, n, m, r, k, wcat, s_w)
        layer.forward(d["x"].cuda())
        layer.backward(d["dy"].cuda(), accumulate=False)
        fq.grad_sqnorm(layer.d_b, ss, layer.ws)
        layers.append((layer, wcat, m, r, k))
    torch.cuda.synchronize()
    total = sum(oracle.sum_squares(np_of(l.d_b)) for l, *_ in layers)
    assert abs(ss.item() - total) <= 1e-12 * total
    coef = oracle.clip_coef(total, 0.3)
    for layer, wcat, m, r, k in layers:
        ea, es = torch.zeros_like(layer.d_b), torch.zeros_like(layer.d_b)
        fq.adamw_delta(layer.d_b, ea, es, layer.delta_buf, 1, sum_sq=ss)
        buf_gpu = layer.delta_buf.clone()
        layer.update()
        torch.cuda.synchronize()
        z = np.zeros((m, r), np.float32)
        _, _, buf_ref = oracle.adamw_delta(np_of(layer.d_b), z, z, z, 1, clip_coef=coef)
        assert relf(np_of(buf_gpu), buf_ref) < 2e-6
        idx_ref, w_ref, after_ref = oracle.proxy_update(np_of(buf_gpu), wcat, m, r, k)
        assert np.array_equal(np_of(layer.idx), idx_ref) and np.array_equal(np_of(layer.wq), w_ref)
        assert np_of(layer.delta_buf).tobytes() == after_ref.tobytes()
