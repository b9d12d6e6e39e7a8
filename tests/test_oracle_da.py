"""Pins of the oracle's gradient of the adapter factor A (LoRA backward equation dL/dA = B^T dL/dO x^T;
appendix "Ablation on matrix A update"): numpy products on operands decoded by a table built here,
PyTorch's CPU autograd through (W + B A) x, an exact integer case, and the SVD's left factor."""
import numpy as np
import torch

import oracle


def _table(fmt):
    """Value of every FP8 code from the format's definition (sign, exponent, mantissa)."""
    eb, mb, bias = (4, 3, 7) if fmt == oracle.E4M3 else (5, 2, 15)
    out = np.zeros(256)
    for c in range(256):
        sgn = -1.0 if c & 0x80 else 1.0
        e = (c >> mb) & ((1 << eb) - 1)
        f = c & ((1 << mb) - 1)
        if fmt == oracle.E4M3 and (c & 0x7F) == 0x7F:
            out[c] = np.nan
        elif fmt == oracle.E5M2 and e == 31:
            out[c] = np.inf * sgn if f == 0 else np.nan
        elif e == 0:
            out[c] = sgn * f * 2.0 ** (1 - bias - mb)
        else:
            out[c] = sgn * (1 + f / (1 << mb)) * 2.0 ** (e - bias)
    return out


def _bf16(v):
    return torch.from_numpy(np.asarray(v, np.float64)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def test_both_products_against_numpy_on_decoded_operands():
    g = np.random.default_rng(5)
    T, n, m, r = 37, 48, 80, 16
    dyq = oracle.fp8_encode(g.normal(size=(T, m)).astype(np.float32) * 100, oracle.E5M2)
    btq = oracle.fp8_encode(g.normal(size=(r, m)).astype(np.float32) * 10, oracle.E4M3)
    xq = oracle.fp8_encode(g.normal(size=(T, n)).astype(np.float32) * 30, oracle.E4M3)
    s_dy, s_b, s_x = np.float32(3.5), np.float32(0.75), np.float32(11.0)
    t5, t4 = _table(oracle.E5M2), _table(oracle.E4M3)
    G = oracle.adapter_inner_grad(dyq, s_dy, btq, s_b)
    want_g = (t5[dyq] @ t4[btq].T) / (float(s_dy) * float(s_b))
    # the double sum is exact here (few bits per term), so G is the bf16 rounding of the numpy product
    assert np.array_equal(G.astype(np.float64), _bf16(want_g))
    dat = oracle.da(xq, s_x, G)
    want = (t4[xq].T @ G.astype(np.float64)) / float(s_x)
    assert np.allclose(dat, want, rtol=1e-13, atol=0)
    rows = np.array([0, 7, 47])
    assert np.array_equal(oracle.da(xq, s_x, G, rows=rows), dat[rows])
    # a transposed operand or a swapped scale would not survive these
    assert not np.allclose(dat, (t4[xq].T @ G.astype(np.float64)) / float(s_b))


def test_agrees_with_autograd_through_the_unmelded_layer():
    """O = (W + B A) x with a loss whose gradient at O is dY: autograd's gradient at A is the equation's
    B^T dY^T X.  Small integers everywhere, so every FP8 cast, the bf16 rounding of G and all sums are exact."""
    g = np.random.default_rng(6)
    T, n, m, r = 24, 32, 48, 16
    X = g.integers(-3, 4, size=(T, n)).astype(np.float64)
    dY = g.integers(-2, 3, size=(T, m)).astype(np.float64)
    B = g.integers(-2, 3, size=(m, r)).astype(np.float64)
    A = torch.tensor(g.integers(-2, 3, size=(r, n)).astype(np.float64), requires_grad=True)
    W = torch.tensor(g.normal(size=(m, n)))
    O = torch.tensor(X) @ (W + torch.tensor(B) @ A).T
    (O * torch.tensor(dY)).sum().backward()
    xq = oracle.fp8_encode(X.astype(np.float32), oracle.E4M3)
    dyq = oracle.fp8_encode(dY.astype(np.float32), oracle.E5M2)
    btq = oracle.fp8_encode(B.T.astype(np.float32), oracle.E4M3)
    G = oracle.adapter_inner_grad(dyq, np.float32(1.0), btq, np.float32(1.0))
    assert np.array_equal(G.astype(np.float64), dY @ B)
    dat = oracle.da(xq, np.float32(1.0), G)
    assert np.array_equal(dat.T, A.grad.numpy())
    assert np.array_equal(dat.T, B.T @ dY.T @ X)
    # scales divide out: with power-of-two scales the result is exactly the unscaled one
    xq2 = oracle.fp8_encode((X * 4).astype(np.float32), oracle.E4M3)
    dyq2 = oracle.fp8_encode((dY * 8).astype(np.float32), oracle.E5M2)
    btq2 = oracle.fp8_encode((B.T * 2).astype(np.float32), oracle.E4M3)
    G2 = oracle.adapter_inner_grad(dyq2, np.float32(8.0), btq2, np.float32(2.0))
    assert np.array_equal(oracle.da(xq2, np.float32(4.0), G2), dat)


def test_inner_gradient_is_rounded_to_sixteen_bits():
    dyq = oracle.fp8_encode(np.array([[1.0, 1.0, 0.0078125]], np.float32), oracle.E5M2)      # 1 + 1 + 2^-7
    btq = oracle.fp8_encode(np.array([[1.0, 1.0, 1.0]], np.float32), oracle.E4M3)
    G = oracle.adapter_inner_grad(dyq, np.float32(1.0), btq, np.float32(1.0))
    assert G[0, 0] == 2.0                                           # 2.0078125 needs nine significant bits: tie to even
    dyq[0, 2] = oracle.fp8_encode(np.array([0.0234375], np.float32), oracle.E5M2)[0]                        # 2 + 3 * 2^-7: rounds up
    assert oracle.adapter_inner_grad(dyq, np.float32(1.0), btq, np.float32(1.0))[0, 0] == 2.03125


def test_left_and_right_factor_multiply_to_the_truncated_matrix():
    g = np.random.default_rng(7)
    m, n, r = 40, 56, 8
    U, _ = np.linalg.qr(g.normal(size=(m, m)))
    V, _ = np.linalg.qr(g.normal(size=(n, n)))
    sv = np.concatenate([np.linspace(10, 3, r), np.full(m - r, 1e-3)])
    E = (U * sv[None, :]) @ V[:m]
    B, A, s = oracle.svd_factors(E, r)
    assert np.allclose(s[:r], sv[:r])
    Er = (U[:, :r] * sv[None, :r]) @ V[:r]
    assert np.allclose(B @ A, Er, atol=1e-10)                        # Eckart-Young: the planted leading part
    assert np.allclose(np.diag(B.T @ B), sv[:r]) and np.allclose(np.diag(A @ A.T), sv[:r])
    A2, _ = oracle.svd_right_factor(E, r)
    assert np.allclose(A2, A)
    # B = E A^T S^-1: the left factor follows from the right one
    assert np.allclose(B, E @ A.T / sv[None, :r], atol=1e-9)
