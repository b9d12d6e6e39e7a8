"""Pins for the oracle's layer functions: melded forward, input gradient, adapter gradient,
proxy-buffer step, row scores, top-k and the row-wise requantizing update.

Each is tied to something other than itself: numpy's matmul on operands decoded with a table
built here from the format definition, exact integer cases, the identities the paper states
(merged-output split, modified LoRA-backward, quantization error as an implicit adapter,
proxy-update algebra) and brute force on tiny inputs.
"""
import itertools

import numpy as np
import pytest

import oracle
import workloads
from test_oracle_fp8 import _brute_force_encode, _value_table

T4 = _value_table(oracle.E4M3)
T5 = _value_table(oracle.E5M2)


def _dec(codes, table):
    lut = np.zeros(256)
    for c, v in table.items():
        lut[c] = v
        lut[c | 0x80] = -v
    return lut[codes]


def _finite_codes(g, shape, fmt):
    c = g.integers(0, 256, size=shape).astype(np.uint8)
    if fmt == oracle.E4M3:
        c[(c & 0x7F) == 0x7F] = 0x3A
    else:
        c[(c & 0x7F) >= 0x7C] = 0x3A
    return c


def _relf(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# ------------------------------------------------------------------ forward -------------

def test_fwd_matches_numpy_matmul_on_decoded_operands():
    g = np.random.default_rng(0)
    T, n, m, r = 19, 45, 23, 5                      # all different, none a tile multiple
    xq = _finite_codes(g, (T, n), oracle.E4M3)
    wq = _finite_codes(g, (m + r, n), oracle.E4M3)
    s_w, s_x = np.float32(3.7), np.float32(0.23)
    got = oracle.melded_fwd(xq, wq, s_w, s_x, m, r)
    want = _dec(xq, T4) @ _dec(wq, T4).T / (np.float64(s_w) * np.float64(s_x))
    assert got.shape == (T, m + r)
    assert _relf(got, want) < 1e-14


def test_fwd_exact_integer_case():
    """Small-integer code values and power-of-two scales: every product and sum is exact."""
    g = np.random.default_rng(1)
    T, n, m, r = 8, 64, 12, 4
    xi = g.integers(-8, 9, size=(T, n))
    wi = g.integers(-8, 9, size=(m + r, n))
    xq = oracle.fp8_encode(xi.astype(np.float32), oracle.E4M3)
    wq = oracle.fp8_encode(wi.astype(np.float32), oracle.E4M3)
    got = oracle.melded_fwd(xq, wq, np.float32(2.0), np.float32(0.5), m, r)
    assert np.array_equal(got, (xi @ wi.T).astype(np.float64))


def test_fwd_identity_weight_returns_dequantized_input():
    g = np.random.default_rng(2)
    n = 16
    xq = _finite_codes(g, (7, n), oracle.E4M3)
    eye = oracle.fp8_encode(np.eye(n, dtype=np.float32), oracle.E4M3)
    wq = np.concatenate([eye, eye[:4]], axis=0)
    s_x = np.float32(5.0)
    got = oracle.melded_fwd(xq, wq, np.float32(1.0), s_x, n, 4)
    assert np.array_equal(got[:, :n], _dec(xq, T4) / 5.0)
    assert np.array_equal(got[:, n:], _dec(xq, T4)[:, :4] / 5.0)


def test_fwd_merged_output_splits_into_the_two_separate_products():
    """Merged-output equation: rows of the concatenated weight act independently."""
    g = np.random.default_rng(3)
    T, n, m, r = 11, 32, 9, 3
    xq = _finite_codes(g, (T, n), oracle.E4M3)
    wq = _finite_codes(g, (m + r, n), oracle.E4M3)
    merged = oracle.melded_fwd(xq, wq, 2.0, 3.0, m, r)
    only_w = oracle.melded_fwd(xq, wq[:m], 2.0, 3.0, m, 0)
    only_a = oracle.melded_fwd(xq, wq[m:], 2.0, 3.0, r, 0)
    assert np.array_equal(merged[:, :m], only_w)
    assert np.array_equal(merged[:, m:], only_a)


def test_fwd_row_and_column_selection():
    g = np.random.default_rng(4)
    T, n, m, r = 13, 24, 10, 2
    xq = _finite_codes(g, (T, n), oracle.E4M3)
    wq = _finite_codes(g, (m + r, n), oracle.E4M3)
    full = oracle.melded_fwd(xq, wq, 1.5, 2.5, m, r)
    rows, cols = [12, 0, 5], [11, 3, 10, 0]
    assert np.array_equal(oracle.melded_fwd(xq, wq, 1.5, 2.5, m, r, rows, cols), full[np.ix_(rows, cols)])
    assert np.array_equal(oracle.melded_fwd(xq, wq, 1.5, 2.5, m, r, rows, None), full[rows])
    assert np.array_equal(oracle.melded_fwd(xq, wq, 1.5, 2.5, m, r, None, cols), full[:, cols])


def test_melded_identity_quantization_error_is_the_adapter():
    """With r = min(m, n) the rank-r SVD of (DQ(W~) - W) is exact, so X (W + B A)^T equals
    X DQ(W~)^T to round-off; the FP8 forward equals that up to the E4M3 rounding of X alone."""
    d = workloads.make_inputs(T=24, n=32, m=32, r=32, seed=77)
    x = d["x"].float().numpy().astype(np.float64)
    w = d["w"].numpy()
    wq, s_w, _ = oracle.quantize(w, oracle.E4M3)
    dq = _dec(wq, T4) / np.float64(s_w)
    u, sv, vt = np.linalg.svd(dq - w.astype(np.float64))
    b_hat, a_hat = u * sv, vt
    assert _relf(x @ (w + b_hat @ a_hat).T, x @ dq.T) < 1e-12
    # quantization error identity: DQ(W~) + (W - DQ(W~)) = W
    assert np.array_equal(dq + (w - dq), w.astype(np.float64))
    f = oracle.layer_fwd(d["x"].float().numpy(), np.concatenate([wq, wq[:0]]), s_w, 32, 0)
    err = _relf(f["merged"], x @ dq.T)
    assert 1e-4 < err < 2.0 ** -4


# ------------------------------------------------------------------ input gradient ------

def test_dx_matches_numpy_matmul_and_ignores_adapter_rows():
    g = np.random.default_rng(5)
    T, n, m, r = 17, 29, 21, 6
    dyq = _finite_codes(g, (T, m), oracle.E5M2)
    wq = _finite_codes(g, (m + r, n), oracle.E4M3)
    s_dy, s_w = np.float32(911.0), np.float32(0.7)
    got = oracle.dx(dyq, wq, s_dy, s_w, m)
    want = _dec(dyq, T5) @ _dec(wq[:m], T4) / (np.float64(s_dy) * np.float64(s_w))
    assert got.shape == (T, n)
    assert _relf(got, want) < 1e-14
    wq2 = wq.copy()
    wq2[m:] = 0x7E
    assert np.array_equal(oracle.dx(dyq, wq2, s_dy, s_w, m), got)
    rows, cols = [3, 16], [28, 0, 7]
    assert np.array_equal(oracle.dx(dyq, wq, s_dy, s_w, m, rows, cols), got[np.ix_(rows, cols)])


def test_dx_exact_integer_case_uses_e5m2_for_the_gradient():
    g = np.random.default_rng(6)
    T, n, m = 5, 16, 32
    gi = g.integers(-4, 5, size=(T, m))              # small integers are exact in E5M2
    wi = g.integers(-8, 9, size=(m, n))
    dyq = oracle.fp8_encode(gi.astype(np.float32), oracle.E5M2)
    wq = oracle.fp8_encode(wi.astype(np.float32), oracle.E4M3)
    assert np.array_equal(oracle.dx(dyq, wq, 4.0, 0.25, m), (gi @ wi).astype(np.float64))
    # the same gradient bytes read as E4M3 would be different numbers
    assert not np.array_equal(_dec(dyq, T4), _dec(dyq, T5))


# ------------------------------------------------------------------ adapter gradient ----

def test_db_matches_numpy_and_quantizes_o_a_with_its_own_scale():
    g = np.random.default_rng(7)
    T, m, r = 33, 14, 6
    dyq = _finite_codes(g, (T, m), oracle.E5M2)
    o_a = oracle.round_bf16(g.normal(size=(T, r)) * 3)
    amax = np.float32(np.abs(o_a).max())
    s_dy = np.float32(123.0)
    got, oaq, s_oa = oracle.db(dyq, s_dy, o_a, amax)
    assert s_oa == np.float32(448.0) / amax
    q_ref, s_ref, _ = oracle.quantize(o_a, oracle.E4M3)
    assert s_ref == s_oa and np.array_equal(oaq, q_ref)
    want = _dec(dyq, T5).T @ _dec(oaq, T4) / (np.float64(s_dy) * np.float64(s_oa))
    assert got.shape == (m, r)
    assert _relf(got, want) < 1e-14
    rows = [13, 2, 2]
    assert np.array_equal(oracle.db(dyq, s_dy, o_a, amax, rows)[0], got[rows])


def test_db_reformulation_identity():
    """dO x^T A^T = dO (A x)^T: the adapter gradient can be formed from the saved A x."""
    g = np.random.default_rng(8)
    T, n, m, r = 12, 20, 9, 4
    dy = _dec(_finite_codes(g, (T, m), oracle.E5M2), T5)
    x = _dec(_finite_codes(g, (T, n), oracle.E4M3), T4)
    a = _dec(_finite_codes(g, (r, n), oracle.E4M3), T4)
    left = (dy.T @ x) @ a.T
    right = dy.T @ (x @ a.T)
    assert _relf(left, right) < 1e-13


def test_db_from_forward_o_a_approximates_full_precision_adapter_gradient():
    """End to end on config-1-like data: dB from (E5M2 dY, E4M3 O_A) tracks dY^T (X A^T)."""
    d = workloads.make_inputs(T=128, n=64, m=48, r=8, seed=5)
    x, w, a, dy = (d[k].float().numpy() for k in ("x", "w", "a", "dy"))
    wq, s_w, _ = oracle.quantize(w, oracle.E4M3)
    aq, _, _ = oracle.quantize(a, oracle.E4M3, scale_in=s_w)
    wcat = np.concatenate([wq, aq])
    f = oracle.layer_fwd(x, wcat, s_w, 48, 8)
    b = oracle.layer_bwd(dy, wcat, s_w, f["o_a"], f["amax_oa"], 48, 8)
    a_dq = _dec(aq, T4) / np.float64(s_w)
    ref = dy.astype(np.float64).T @ (x.astype(np.float64) @ a_dq.T)
    assert _relf(b["db"], ref) < 0.08
    ref_dx = dy.astype(np.float64) @ (_dec(wq, T4) / np.float64(s_w))
    assert _relf(b["dx"], ref_dx) < 0.12


def test_db_wide_matches_numpy_exact_case_and_the_e4m3_variant_on_representable_o_a():
    g = np.random.default_rng(17)
    T, m, r = 37, 11, 5
    dyq = _finite_codes(g, (T, m), oracle.E5M2)
    o_a = oracle.round_bf16(g.normal(size=(T, r)) * 3)
    s_dy = np.float32(77.0)
    got = oracle.db_wide(dyq, s_dy, o_a)
    want = _dec(dyq, T5).T @ o_a.astype(np.float64) / np.float64(s_dy)
    assert got.shape == (m, r) and _relf(got, want) < 1e-14
    rows = [10, 0, 3]
    assert np.array_equal(oracle.db_wide(dyq, s_dy, o_a, rows), got[rows])
    # small integers, power-of-two scale: exact
    dy_small = np.array([[1, -2], [3, 0], [-1, 1]], np.float32)                          # [T=3, m=2]
    oa_small = np.array([[2, 1, 0], [1, -1, 4], [0, 3, -2]], np.float32)                 # [T=3, r=3]
    q5 = oracle.fp8_encode(dy_small * 4, oracle.E5M2)                                    # s_dy = 4
    exact = oracle.db_wide(q5, np.float32(4.0), oa_small)
    assert np.array_equal(exact, dy_small.astype(np.float64).T @ oa_small.astype(np.float64))
    # an O_A that E4M3 represents exactly at its own scale: both variants must agree
    codes = _finite_codes(g, (T, r), oracle.E4M3)
    codes[0, 0] = 0x7E                                                                   # amax maps to 448: s_oa = 1
    o_rep = _dec(codes, T4).astype(np.float32)
    narrow, oaq, s_oa = oracle.db(dyq, s_dy, o_rep, np.float32(448.0))
    assert s_oa == 1.0 and np.array_equal(oaq & 0x7F, codes & 0x7F)
    assert _relf(oracle.db_wide(dyq, s_dy, o_rep), narrow) < 1e-14


def test_db_wide_is_closer_to_the_unquantized_adapter_gradient():
    d = workloads.make_inputs(T=256, n=64, m=48, r=8, seed=9)
    x, w, a, dy = (d[k].float().numpy() for k in ("x", "w", "a", "dy"))
    wq, s_w, _ = oracle.quantize(w, oracle.E4M3)
    aq, _, _ = oracle.quantize(a, oracle.E4M3, scale_in=s_w)
    wcat = np.concatenate([wq, aq])
    f = oracle.layer_fwd(x, wcat, s_w, 48, 8)
    b = oracle.layer_bwd(dy, wcat, s_w, f["o_a"], f["amax_oa"], 48, 8)
    wide = oracle.db_wide(b["dyq"], b["s_dy"], f["o_a"])
    ref = _dec(b["dyq"], T5).T @ f["o_a"].astype(np.float64) / np.float64(b["s_dy"])
    assert _relf(wide, ref) < 1e-14
    # against the same E5M2 gradient times the fp64 O_A before its bf16 rounding
    o_exact = (_dec(f["xq"], T4) @ _dec(aq, T4).T) / (np.float64(f["s_x"]) * np.float64(s_w))
    ideal = _dec(b["dyq"], T5).T @ o_exact / np.float64(b["s_dy"])
    assert _relf(wide, ideal) < _relf(b["db"], ideal)
    assert _relf(wide, ideal) < 4e-3


def test_delta_accumulate_closed_form():
    buf = np.array([[0.0, 1.0], [-2.0, 1e-3]], np.float32)
    d_b = np.array([[10.0, -5.0], [0.5, 1.0 / 3.0]], np.float64)
    lr = np.float32(2e-4)
    got = oracle.delta_accumulate(buf, d_b, lr)
    want = buf + (-lr * d_b.astype(np.float32)).astype(np.float32)
    assert np.array_equal(got, want.astype(np.float32))
    # exact case: lr = 2^-12, dB = 8 and -3  ->  steps -2^-9 and +3*2^-12
    got2 = oracle.delta_accumulate(np.float32([[1.0, 0.5]]), np.float64([[8.0, -3.0]]), np.float32(2.0 ** -12))
    assert got2[0, 0] == 1.0 - 2.0 ** -9 and got2[0, 1] == 0.5 + 3 * 2.0 ** -12
    assert np.array_equal(buf, np.array([[0.0, 1.0], [-2.0, 1e-3]], np.float32))     # input untouched


# ------------------------------------------------------------------ scores and top-k ----

def test_row_scores_are_l1_norms():
    g = np.random.default_rng(9)
    buf = g.normal(size=(40, 16)).astype(np.float32)
    want = np.abs(buf.astype(np.float64)).sum(axis=1)
    assert np.allclose(oracle.row_scores(buf), want, rtol=1e-15, atol=0)
    assert oracle.row_scores(np.array([[1.0, -2.0, 3.5]], np.float32))[0] == 6.5


def _brute_topk(score, k):
    order = sorted(range(len(score)), key=lambda i: (-score[i], i))
    return order[:k]


def test_topk_brute_force_all_k_with_ties():
    g = np.random.default_rng(10)
    for m in (1, 2, 5, 17, 64):
        score = g.integers(0, 6, size=m).astype(np.float64)       # many ties
        for k in range(1, m + 1):
            assert list(oracle.topk_rows(score, k)) == _brute_topk(score, k)
    score = np.array([3.0, 7.0, 7.0, 1.0, 7.0, 3.0])
    assert list(oracle.topk_rows(score, 4)) == [1, 2, 4, 0]
    assert list(oracle.topk_rows(np.zeros(9), 3)) == [0, 1, 2]


def test_topk_is_a_max_not_a_min_and_uses_magnitudes():
    buf = np.zeros((6, 4), np.float32)
    buf[4] = [-5, -5, -5, -5]        # largest in magnitude, negative entries
    buf[1] = [1, 1, 1, 1]
    buf[2] = [3, -3, 0, 0]
    idx, _, _ = oracle.proxy_update(buf, np.zeros((6 + 4, 8), np.uint8), 6, 4, 3)
    assert list(idx) == [4, 2, 1]


# ------------------------------------------------------------------ row update ----------

def _update_case(seed, n=40, m=24, r=4, k=5, scale=0.5):
    g = np.random.default_rng(seed)
    wq = _finite_codes(g, (m + r, n), oracle.E4M3)
    buf = (g.normal(size=(m, r)) * scale * np.exp(g.normal(size=(m, 1)))).astype(np.float32)
    return wq, buf, n, m, r, k


def test_update_rows_brute_force():
    wq, buf, n, m, r, k = _update_case(11)
    idx, w_new, b_new = oracle.proxy_update(buf, wq, m, r, k)
    assert list(idx) == _brute_topk(np.abs(buf.astype(np.float64)).sum(1), k)
    a_val = _dec(wq[m:], T4)
    for i in range(m):
        if i not in idx:
            assert np.array_equal(w_new[i], wq[i])
            assert np.array_equal(b_new[i], buf[i])
            continue
        target = _dec(wq[i], T4) + buf[i].astype(np.float64) @ a_val
        for j in range(n):
            want = _brute_force_encode(np.float32(target[j]), oracle.E4M3, T4)
            # the accumulation order can move the fp64 sum by an ulp; only exact ties could differ
            assert w_new[i, j] == want or abs(_dec(np.uint8(w_new[i, j]), T4) - target[j]) <= abs(_dec(np.uint8(want), T4) - target[j]) * (1 + 1e-12)
        assert np.all(b_new[i] == 0) and not np.any(np.signbit(b_new[i]))
    assert np.array_equal(w_new[m:], wq[m:])                # adapter rows never change


def test_update_with_zero_buffer_only_normalises_negative_zero():
    wq, buf, n, m, r, k = _update_case(12)
    buf[:] = 0
    wq[0, :4] = [0x80, 0x00, 0x81, 0xFE]
    idx, w_new, _ = oracle.proxy_update(buf, wq, m, r, k)
    assert list(idx) == list(range(k))
    want = wq.copy()
    for i in range(k):
        want[i][want[i] == 0x80] = 0x00                      # -0 + (+0) = +0
    assert np.array_equal(w_new, want)


def test_update_half_ulp_and_proxy_algebra():
    """Each new code is the nearest E4M3 value to dec(W~) + dB A~ (or the clipped extreme):
    W + (B + dB) A = (W + B A) + dB A, applied on code values because the scale cancels."""
    wq, buf, n, m, r, k = _update_case(13, scale=2.0)
    idx, w_new, _ = oracle.proxy_update(buf, wq, m, r, k)
    vals = np.array(sorted(T4.values()))
    a_val = _dec(wq[m:], T4)
    moved = 0
    for i in idx:
        target = _dec(wq[i], T4) + buf[i].astype(np.float64) @ a_val
        new = _dec(w_new[i], T4)
        clipped = np.clip(target, -448, 448)
        pos = np.searchsorted(vals, np.abs(clipped))
        lo, hi = vals[np.maximum(pos - 1, 0)], vals[np.minimum(pos, len(vals) - 1)]
        half = np.maximum(hi - lo, 2.0 ** -9) / 2
        assert np.all(np.abs(new - clipped) <= half * (1 + 1e-6))
        moved += int(np.sum(w_new[i] != wq[i]))
    assert moved > 0


def test_update_keep_buffer_when_not_clearing():
    wq, buf, n, m, r, k = _update_case(14)
    idx1, w1, b1 = oracle.proxy_update(buf, wq, m, r, k, clear_selected=False)
    idx2, w2, b2 = oracle.proxy_update(buf, wq, m, r, k, clear_selected=True)
    assert np.array_equal(idx1, idx2) and np.array_equal(w1, w2)
    assert np.array_equal(b1, buf)
    assert np.all(b2[idx2] == 0)
    mask = np.ones(m, bool)
    mask[idx2] = False
    assert np.array_equal(b2[mask], buf[mask])


def test_update_sign_of_the_step():
    """A positive buffer entry against a positive adapter entry must raise the weight."""
    n, m, r = 4, 2, 1
    wq = np.zeros((m + r, n), np.uint8)
    wq[0] = oracle.fp8_encode(np.float32([8, 8, 8, 8]), 0)
    wq[2] = oracle.fp8_encode(np.float32([1, -1, 2, 0]), 0)
    buf = np.array([[4.0], [0.0]], np.float32)
    idx, w_new, _ = oracle.proxy_update(buf, wq, m, r, 1)
    assert list(idx) == [0]
    assert list(_dec(w_new[0], T4)) == [12.0, 4.0, 16.0, 8.0]
    assert np.array_equal(w_new[1], wq[1])


def test_config1_end_to_end_shapes_and_sanity():
    d = workloads.config_layer_inputs(1)
    c = d["config"]
    m, n, r = d["shape"].m, d["shape"].n, c.r
    x, w, a, dy = (d[k].float().numpy() for k in ("x", "w", "a", "dy"))
    wq, s_w, _ = oracle.quantize(w, oracle.E4M3)
    aq, _, _ = oracle.quantize(a, oracle.E4M3, scale_in=s_w)
    wcat = np.concatenate([wq, aq])
    f = oracle.layer_fwd(x, wcat, s_w, m, r)
    assert f["y"].shape == (c.T, m) and f["o_a"].shape == (c.T, r)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert _relf(f["y"], ref) < 0.06
    b = oracle.layer_bwd(dy, wcat, s_w, f["o_a"], f["amax_oa"], m, r,
                         delta_buf=np.zeros((m, r), np.float32), lr=c.lr)
    idx, w_new, buf_new = oracle.proxy_update(b["delta_buf"], wcat, m, r, c.k)
    assert len(set(idx.tolist())) == c.k
    assert np.all(buf_new[idx] == 0)
