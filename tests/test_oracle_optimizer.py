"""Pins of the oracle's optimizer step (AdamW into the proxy buffer, gradient-norm clipping)
against things other than itself: PyTorch's CPU AdamW and clip_grad_norm_, closed forms of the
first step, and invariants."""
import numpy as np
import torch

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


def test_matches_torch_adamw_with_clipping_over_several_steps_and_layers():
    """Two 'layers' trained for 6 steps with torch.optim.AdamW(weight_decay=0) in fp64 and
    clip_grad_norm_(0.3) over both; the oracle's buffers must track B - B_0 (no row is folded
    into the weight here, so the buffer is the whole change of B)."""
    g = _rng(0)
    shapes = [(48, 16), (32, 64)]
    params = [torch.zeros(s, dtype=torch.float64, requires_grad=True) for s in shapes]
    opt = torch.optim.AdamW(params, lr=2e-4, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0)
    state = [(np.zeros(s, np.float32), np.zeros(s, np.float32), np.zeros(s, np.float32)) for s in shapes]
    for step in range(1, 7):
        scale = [0.01, 1.0, 30.0, 1e-4, 0.3, 5.0][step - 1]          # below and above the clipping threshold
        grads = [(g.normal(size=s) * scale).astype(np.float32) for s in shapes]
        for p, gr in zip(params, grads):
            p.grad = torch.from_numpy(gr.astype(np.float64))
        torch.nn.utils.clip_grad_norm_(params, 0.3)
        opt.step()
        coef = oracle.clip_coef(sum(oracle.sum_squares(gr) for gr in grads), 0.3)
        state = [oracle.adamw_delta(gr, m, v, b, step, clip_coef=coef) for gr, (m, v, b) in zip(grads, state)]
        for p, (m, v, b) in zip(params, state):
            ref = p.detach().numpy()
            assert np.max(np.abs(b - ref)) <= 2e-6 * np.max(np.abs(ref)) + 1e-12
            st = opt.state[p]
            # the oracle keeps fp32 moments (torch here fp64): agreement to fp32 rounding of the larger terms
            for mine, theirs in ((m, st["exp_avg"].numpy()), (v, st["exp_avg_sq"].numpy())):
                assert np.max(np.abs(mine - theirs)) <= 1e-6 * np.max(np.abs(theirs))


def test_first_step_closed_form():
    """t = 1, zero moments: m/(1-b1) = g and v/(1-b2) = g^2, so the change is -lr * g / (|g| + eps)."""
    gr = np.array([[0.5, -2.0, 1e-3, -1e-10, 0.0, 3e4]], np.float32)
    z = np.zeros_like(gr)
    buf0 = np.array([[1.0, -1.0, 0.0, 0.0, 0.25, 0.0]], np.float32)
    m, v, b = oracle.adamw_delta(gr, z, z, buf0, 1, lr=1e-2, eps=1e-8)
    g64 = gr.astype(np.float64)
    want = buf0 + (-1e-2 * g64 / (np.abs(g64) + 1e-8))
    assert np.array_equal(b, want.astype(np.float32))
    assert np.allclose(m, 0.1 * g64, rtol=1e-7) and np.allclose(v, 0.001 * g64 * g64, rtol=1e-7)
    assert b[0, 4] == 0.25                                           # zero gradient: no change


def test_zero_gradient_decays_moments_and_moves_with_momentum_only():
    m0 = np.full((4, 16), 0.5, np.float32)
    v0 = np.full((4, 16), 0.25, np.float32)
    z = np.zeros((4, 16), np.float32)
    m, v, b = oracle.adamw_delta(z, m0, v0, z, 10)
    assert np.allclose(m, 0.45) and np.allclose(v, 0.25 * 0.999)
    want = -(2e-4 / (1 - 0.9 ** 10)) * 0.45 / (np.sqrt(0.25 * 0.999) / np.sqrt(1 - 0.999 ** 10) + 1e-8)
    assert np.allclose(b, want, rtol=1e-6)


def test_clip_coefficient():
    assert oracle.clip_coef(0.0, 0.3) == 1.0
    assert oracle.clip_coef(0.3 ** 2 * 0.99, 0.3) == 1.0             # below the threshold: untouched
    c = oracle.clip_coef(100.0, 0.3)                                  # norm 10
    assert abs(c - 0.3 / (10.0 + 1e-6)) < 1e-15
    g = _rng(3).normal(size=(20, 16)).astype(np.float32) * 7
    ss = oracle.sum_squares(g)
    assert abs(ss - float(np.sum(g.astype(np.float64) ** 2))) <= 1e-12 * ss
    clipped = g.astype(np.float64) * oracle.clip_coef(ss, 0.3)
    assert abs(np.linalg.norm(clipped) - 0.3) < 1e-6


def test_buffer_accumulates_across_steps():
    """Two steps from the same state: the buffer after the second step is the first result plus
    the second change (it stores the accumulated change of B)."""
    g = _rng(5)
    g1, g2 = (g.normal(size=(8, 16)).astype(np.float32) for _ in range(2))
    z = np.zeros((8, 16), np.float32)
    m1, v1, b1 = oracle.adamw_delta(g1, z, z, z, 1)
    m2, v2, b2 = oracle.adamw_delta(g2, m1, v1, b1, 2)
    _, _, only2 = oracle.adamw_delta(g2, m1, v1, z, 2)
    assert np.allclose(b2, b1 + only2, rtol=0, atol=1e-10)
    assert np.all(np.sign(b1) == -np.sign(g1))
