"""Pins of the oracle's initialization steps (residual, rank-r factor) against the mathematics."""
import numpy as np

import oracle


def _w(m, n, seed):
    return (np.random.default_rng(seed).normal(size=(m, n)) * 0.02).astype(np.float32)


def test_residual_is_the_dequantization_error_and_is_bounded_by_half_a_step():
    w = _w(48, 64, 1)
    wq, s_w, _ = oracle.quantize(w, oracle.E4M3)
    e = oracle.init_residual(w, wq, s_w)
    dq = oracle.fp8_decode(wq, oracle.E4M3) / np.float64(s_w)
    assert np.max(np.abs(e - (dq - w))) <= 1e-9                      # fp32 roundings of the two operations only
    # |error| <= half the spacing of the E4M3 grid at that magnitude (relative 2^-4), or half a subnormal step
    bound = np.maximum(np.abs(w) * 2.0 ** -4, 2.0 ** -10 / np.float64(s_w)) * 1.001
    assert np.all(np.abs(e) <= bound)
    assert np.any(e > 0) and np.any(e < 0)


def test_residual_exact_cases():
    w = np.array([[1.0, 0.5, -0.25, 0.0, 3.0, -7.0, 448.0, 0.001]], np.float32)
    wq = oracle.fp8_encode(w * 1.0, oracle.E4M3)
    e = oracle.init_residual(w, wq, np.float32(1.0))
    # representable values leave no residual; 0.001 rounds to the subnormal grid (step 2^-9): 0.001 -> 2^-9 * 1 = 0.001953125
    assert np.array_equal(e[0, :7], np.zeros(7, np.float32))
    assert e[0, 7] == np.float32(np.float32(2.0 ** -9) - np.float32(0.001))
    e2 = oracle.init_residual(w * 0.5, wq, np.float32(2.0))         # scale 2: same codes, values halved
    assert np.array_equal(e2[0, :7], np.zeros(7, np.float32))


def test_rank_r_factor_is_the_best_rank_r_approximation():
    g = np.random.default_rng(3)
    e = g.normal(size=(40, 56))
    r = 6
    a, sv = oracle.svd_right_factor(e, r)
    assert a.shape == (r, 56)
    # rows of A are orthogonal with squared norms S_i (A = sqrt(S) V^T)
    gram = a @ a.T
    assert np.allclose(gram, np.diag(sv[:r]), atol=1e-10)
    # the matching B = E A^T S^-1 reconstructs with the Eckart-Young error sqrt(sum of the other S^2)
    b = e @ a.T / sv[:r]
    err = np.linalg.norm(e - b @ a)
    assert abs(err - np.sqrt(np.sum(sv[r:] ** 2))) < 1e-9
    # no other rank-r subspace does better: random ones are worse
    for _ in range(5):
        q, _ = np.linalg.qr(g.normal(size=(56, r)))
        assert np.linalg.norm(e - e @ q @ q.T) >= err - 1e-12


def test_planted_low_rank_matrix_is_recovered():
    g = np.random.default_rng(4)
    r = 4
    left, right = g.normal(size=(30, r)), g.normal(size=(r, 50))
    e = left @ right
    a, sv = oracle.svd_right_factor(e, r)
    assert np.all(sv[r:] < 1e-10 * sv[0])
    proj = a.T @ np.linalg.solve(a @ a.T, a)                         # projector on the row space of A
    assert np.allclose(right @ proj, right, atol=1e-9)               # it contains the planted row space


def test_init_adapter_sign_and_identity():
    """DQ(W~) = W + E exactly in the oracle's arithmetic, and B^ A^ with B^ = E A^T S^-1 is the rank-r part of
    E: the quantized backbone reads as W + B^ A^ + (what rank r cannot hold)."""
    w = _w(64, 96, 7)
    r = 8
    d = oracle.init_adapter(w, r)
    dq = (oracle.fp8_decode(d["wq"], oracle.E4M3) / np.float64(d["s_w"])).astype(np.float32)
    assert np.max(np.abs((w + d["e"]) - dq)) <= 2e-9
    a = d["a_hat"]
    b = d["e"].astype(np.float64) @ a.T / d["sv"][:r]
    tail = np.linalg.norm(d["e"] - b @ a)
    assert abs(tail - np.sqrt(np.sum(d["sv"][r:] ** 2))) < 1e-9
    assert tail < np.linalg.norm(d["e"])                             # the adapter explains part of the error
    # A~ is A^ cast with the backbone's scale
    ref, _, _ = oracle.quantize(a.astype(np.float32), oracle.E4M3, scale_in=d["s_w"])
    assert np.array_equal(d["a_q"], ref)
