"""GPU parity of the initialization steps against the CPU oracle.

The residual is bit-exact.  The rank-r factor is the result of an iteration whose limit (the
truncated SVD) is unique only as a subspace and only up to the sign of each vector, so what is
compared is what is unique: the projector on the row space, the singular values and the energy
captured, with the exact SVD of the oracle as reference; what is not unique is checked for
validity (orthogonal rows, squared norms equal to the Ritz values, Ritz values = |E v|).

Tolerances.  With a spectral gap the subspace iteration converges at (sigma_{l+1}/sigma_r)^(2q+1);
the planted cases have a gap of 10^2 or more, so after q = 3 rounds what remains is fp32 rounding
of products over n terms: 1e-4 on projector and singular values.  Quantization residuals have no
gap; there the r Ritz values must capture at least 90 % of the energy of the best rank-r factor."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
from gpu_common import np_of

pytestmark = pytest.mark.gpu


def _factor(e: np.ndarray, r: int, iters: int, seed: int = 0):
    m, n = e.shape
    g = torch.Generator().manual_seed(seed)
    omega = torch.randn(r + 8, n, generator=g).cuda()
    a = torch.empty(r, n, dtype=torch.float32, device="cuda")
    sig = torch.empty(r, dtype=torch.float32, device="cuda")
    ws = torch.empty(fq.svd_workspace_bytes(m, n, r), dtype=torch.uint8, device="cuda")
    fq.svd_right_factor(torch.from_numpy(e).cuda(), r, omega, iters, a, sig, ws)
    torch.cuda.synchronize()
    return np_of(a).astype(np.float64), np_of(sig).astype(np.float64)


def _projector(a):
    q, _ = np.linalg.qr(a.T)
    return q @ q.T


@pytest.mark.parametrize("m,n", [(64, 128), (300, 400), (1000, 520), (4096, 1024)])
def test_residual_bit_exact(m, n):
    w = (np.random.default_rng(m).normal(size=(m, n)) * 0.02).astype(np.float32)
    w[0, :4] = [0.0, -0.0, 1e-9, 0.09]
    wq, s_w, _ = oracle.quantize(w, oracle.E4M3)
    ref = oracle.init_residual(w, wq, s_w)
    e = torch.empty(m, n, dtype=torch.float32, device="cuda")
    fq.init_residual(torch.from_numpy(w).cuda(), torch.from_numpy(wq).cuda(), torch.tensor([s_w], device="cuda"), e)
    torch.cuda.synchronize()
    assert np_of(e).tobytes() == ref.tobytes()


@pytest.mark.parametrize("m,n,r", [(300, 400, 16), (520, 272, 24), (1024, 2048, 64), (200, 1000, 120)])
def test_factor_of_a_matrix_with_a_spectral_gap(m, n, r):
    g = np.random.default_rng(m + n)
    u, _ = np.linalg.qr(g.normal(size=(m, r)))
    v, _ = np.linalg.qr(g.normal(size=(n, r)))
    s = np.linspace(10.0, 2.0, r)                                   # distinct, well separated from the noise
    e = ((u * s) @ v.T + 1e-3 * g.normal(size=(m, n)) / np.sqrt(max(m, n))).astype(np.float32)
    print(f"gap case m={m} n={n} r={r}", flush=True)
    a, sig = _factor(e, r, iters=3, seed=r)
    a_ref, sv = oracle.svd_right_factor(e, r)
    assert np.max(np.abs(sig - sv[:r])) <= 1e-4 * sv[0]
    assert np.all(np.diff(sig) <= 0)
    gram = a @ a.T
    assert np.max(np.abs(gram - np.diag(sig))) <= 1e-4 * sig[0]     # orthogonal rows, squared norms sigma_i
    assert np.linalg.norm(_projector(a) - _projector(a_ref)) <= 1e-3
    # each row is +/- the oracle's row (distinct singular values): compare up to sign
    for i in range(r):
        c = float(a[i] @ a_ref[i]) / (np.linalg.norm(a[i]) * np.linalg.norm(a_ref[i]))
        assert abs(abs(c) - 1.0) <= 1e-4, (i, c)
    # Ritz values are |E v_i|
    ev = e.astype(np.float64) @ (a / np.sqrt(sig)[:, None]).T
    assert np.max(np.abs(np.linalg.norm(ev, axis=0) - sig)) <= 1e-4 * sig[0]


def test_factor_of_a_quantization_residual_and_the_layer_it_initializes():
    """Initialization algorithm end to end on the GPU: Q(W), residual, rank-r factor, cast with s_w."""
    m, n, r, k = 1024, 768, 32, 8
    g = np.random.default_rng(11)
    w = (g.normal(size=(m, n)) * 0.02).astype(np.float32)
    ref = oracle.init_adapter(w, r)
    layer = fq.MeldedLinear(64, n, m, r, k)
    wg = torch.from_numpy(w).cuda()
    fq.quantize(wg, fq.E4M3, layer.wq[:m], layer.s_w, layer.ws)
    e = torch.empty(m, n, dtype=torch.float32, device="cuda")
    fq.init_residual(wg, layer.wq[:m], layer.s_w, e)
    torch.cuda.synchronize()
    assert np.array_equal(np_of(layer.wq[:m]), ref["wq"]) and np_of(e).tobytes() == ref["e"].tobytes()
    a, sig = _factor(ref["e"], r, iters=8, seed=5)
    sv = ref["sv"]
    assert np.all(sig <= sv[:r] * (1 + 1e-4))                        # Ritz values approach from below
    captured, best = float(np.sum(sig ** 2)), float(np.sum(sv[:r] ** 2))
    print(f"captured {captured / best:.4f} of the best rank-{r} energy", flush=True)
    assert captured >= 0.90 * best
    gram = a @ a.T
    assert np.max(np.abs(gram - np.diag(sig))) <= 1e-4 * sig[0]
    ev = ref["e"].astype(np.float64) @ (a / np.sqrt(sig)[:, None]).T
    assert np.max(np.abs(np.linalg.norm(ev, axis=0) - sig)) <= 1e-4 * sig[0]
    # last step of the initialization: the cast of A^ with the backbone's scale equals the oracle's cast of the same A^
    a32 = torch.from_numpy(a.astype(np.float32)).cuda()
    s_tmp = torch.zeros(1, device="cuda")
    fq.quantize(a32, fq.E4M3, layer.wq[m:], s_tmp, layer.ws, scale_in=layer.s_w)
    torch.cuda.synchronize()
    aq_ref, _, _ = oracle.quantize(a.astype(np.float32), oracle.E4M3, scale_in=ref["s_w"])
    assert np.array_equal(np_of(layer.wq[m:]), aq_ref)
    # and the layer it initializes runs: O_A = A~ x
    x = torch.randn(64, n, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16)
    layer.forward(x.cuda())
    torch.cuda.synchronize()
    f = oracle.layer_fwd(x.float().numpy(), np_of(layer.wq), ref["s_w"], m, r)
    assert np.linalg.norm(np_of(layer.o_a) - f["o_a"]) <= 1e-3 * np.linalg.norm(f["o_a"])
