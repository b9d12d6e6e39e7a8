"""The method end to end on a synthetic regression: gradients into the proxy buffer, top-k rows folded
into the FP8 backbone every step.  The layer has no trainable tensor other than the buffer, so a
falling loss shows that the folded rows really carry the adapter's learning.  The same loop on the
CPU oracle gives the trajectory to compare with."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_24061_amd.nn import MeldedLoRALinear

pytestmark = pytest.mark.gpu

T, N, M, R, K = 512, 256, 256, 16, 64
LR, STEPS = 0.25, 60


def _problem():
    g = np.random.default_rng(0)
    w = (g.normal(size=(M, N)) * 0.02).astype(np.float32)
    a = (g.normal(size=(R, N)) / R).astype(np.float32)
    wq, s_w, _ = oracle.quantize(w, oracle.E4M3)
    aq, _, _ = oracle.quantize(a, oracle.E4M3, scale_in=s_w)
    a_dq = oracle.fp8_decode(aq, oracle.E4M3) / np.float64(s_w)
    w_dq = oracle.fp8_decode(wq, oracle.E4M3) / np.float64(s_w)
    b_star = g.normal(size=(M, R))
    b_star *= 0.5 * np.linalg.norm(w_dq) / np.linalg.norm(b_star @ a_dq)       # teacher: backbone + half its norm
    w_teacher = (w_dq + b_star @ a_dq).astype(np.float32)
    xs = [oracle.round_bf16(np.random.default_rng(100 + s).normal(size=(T, N))).astype(np.float32) for s in range(STEPS)]
    return w, a, np.concatenate([wq, aq]), s_w, w_teacher, xs


def _oracle_losses(wcat, s_w, w_teacher, xs, steps):
    wc, buf, losses = wcat.copy(), np.zeros((M, R), np.float32), []
    for x in xs[:steps]:
        f = oracle.layer_fwd(x, wc, s_w, M, R)
        y = oracle.round_bf16(f["y"]).astype(np.float64)
        y_t = (x @ w_teacher.T).astype(np.float64)
        losses.append(0.5 * np.mean(np.sum((y - y_t) ** 2, axis=1)))
        dy = oracle.round_bf16((y - y_t) / T).astype(np.float32)
        b = oracle.layer_bwd(dy, wc, s_w, f["o_a"], f["amax_oa"], M, R, delta_buf=buf, lr=np.float32(LR))
        _, wc, buf = oracle.proxy_update(b["delta_buf"], wc, M, R, K)
    return losses


def test_loss_falls_and_tracks_the_oracle_loop():
    w, a, wcat, s_w, w_teacher, xs = _problem()
    layer = MeldedLoRALinear(N, M, R, K, sgd_lr=LR)
    layer.load_weights(torch.from_numpy(w).cuda(), torch.from_numpy(a).cuda())
    assert np.array_equal(layer.wq.cpu().numpy(), wcat)
    wt = torch.from_numpy(w_teacher).cuda()
    losses = []
    for x_np in xs:
        x = torch.from_numpy(x_np).cuda().to(torch.bfloat16).requires_grad_(True)
        y = layer(x).float()
        y_t = x.detach().float() @ wt.T
        loss = 0.5 * ((y - y_t) ** 2).sum(dim=1).mean()
        loss.backward()                                  # dY = (y - y_t) / T; the buffer step happens in backward
        layer.proxy_update()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.06 * losses[0], losses[::10]
    assert min(losses) == pytest.approx(losses[-1], rel=0.5)          # it stays down, no late blow-up
    # the first steps follow the CPU loop closely (later ones drift apart through bf16 rounding flips)
    ref = _oracle_losses(wcat, s_w, w_teacher, xs, 6)
    for got, want in zip(losses[:6], ref):
        assert got == pytest.approx(want, rel=0.03), (losses[:6], ref)


def test_nothing_learned_without_folding():
    """Control: the forward reads only the FP8 backbone, so with the buffer never folded the loss stays put."""
    w, a, wcat, s_w, w_teacher, xs = _problem()
    layer = MeldedLoRALinear(N, M, R, K, sgd_lr=LR)
    layer.load_weights(torch.from_numpy(w).cuda(), torch.from_numpy(a).cuda())
    wt = torch.from_numpy(w_teacher).cuda()
    losses = []
    for x_np in xs[:10]:
        x = torch.from_numpy(x_np).cuda().to(torch.bfloat16).requires_grad_(True)
        y = layer(x).float()
        loss = 0.5 * ((y - x.detach().float() @ wt.T) ** 2).sum(dim=1).mean()
        loss.backward()
        losses.append(float(loss.detach()))
    assert max(losses) < 1.15 * min(losses)
    assert np.array_equal(layer.wq.cpu().numpy(), wcat)
    assert float(layer.delta_buf.abs().sum()) > 0
